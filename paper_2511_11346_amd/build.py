"""Builds libmtpc.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["unembed.hip", "grad.hip", "circuits.hip", "speculative.hip", "backward.hip", "api.hip"]
OUT = os.path.join(HERE, "libmtpc.so")


def build(verbose: bool = False) -> str:
    """Compile every translation unit (in parallel) and link libmtpc.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["-fPIC", "--offload-arch=gfx950", "-O3", "-std=c++17",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def run(cmd):
        res = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass does not know the device-only target feature and says so: harmless
        err = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "is not a recognized feature" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + err)
        if verbose and err.strip():
            print(err, file=sys.stderr)

    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as pool:
        list(pool.map(lambda so: run([hipcc, "-c", *flags, os.path.join(HERE, "csrc", so[0]), "-o", so[1]]),
                      zip(SOURCES, objs)))
    run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", OUT])
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
