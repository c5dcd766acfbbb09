"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before launching."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_11346_amd", "libmtpc.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libmtpc.so not built")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mtpc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mtpc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    from paper_2511_11346_amd import binding
    names = declared_symbols()
    assert len(names) == 39 and sorted(binding.EXPORTS) == names
    L = C.CDLL(LIB)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    from paper_2511_11346_amd import binding
    L = binding.lib()
    assert L.mtpc_status_string(0) == b"ok"
    assert len({L.mtpc_status_string(i) for i in range(6)}) == 6


def _head(**kw):
    from paper_2511_11346_amd.binding import mtpc_head
    hd = mtpc_head()
    hd.B, hd.d, hd.n, hd.r, hd.v, hd.dtype = 4, 64, 4, 2, 16, 1
    hd.h, hd.ld_h, hd.W, hd.Wsum = 0x1000, 64, 0x2000, 0x3000
    hd.workspace, hd.workspace_bytes = 0x10000, 1 << 30
    for k, v in kw.items():
        setattr(hd, k, v)
    return hd


def test_argument_errors_are_reported_without_launching():
    from paper_2511_11346_amd import binding
    L = binding.lib()
    tg, out = C.c_void_p(0x4000), C.c_void_p(0x5000)
    NULL, SHAPE, UNSUP, WS = 1, 2, 3, 4
    assert L.mtpc_cp_loglik(None, tg, out) == NULL
    assert L.mtpc_cp_loglik(C.byref(_head()), None, out) == NULL
    assert L.mtpc_cp_loglik(C.byref(_head(h=None)), tg, out) == NULL
    assert L.mtpc_cp_loglik(C.byref(_head(Wsum=None)), tg, out) == NULL
    assert L.mtpc_cp_loglik(C.byref(_head(B=0)), tg, out) == SHAPE
    assert L.mtpc_cp_loglik(C.byref(_head(ld_h=32)), tg, out) == SHAPE
    assert L.mtpc_ff_loglik(C.byref(_head(r=2)), tg, out) == SHAPE
    assert L.mtpc_cp_loglik(C.byref(_head(d=48)), tg, out) == UNSUP
    assert L.mtpc_cp_loglik(C.byref(_head(v=321)), tg, out) == UNSUP
    assert L.mtpc_cp_loglik(C.byref(_head(r=129)), tg, out) == UNSUP
    assert L.mtpc_cp_loglik(C.byref(_head(dtype=7)), tg, out) == UNSUP
    assert L.mtpc_cp_loglik(C.byref(_head(h=0x1004)), tg, out) == UNSUP
    assert L.mtpc_cp_loglik(C.byref(_head(ld_h=(1 << 23) + 8)), tg, out) == UNSUP     # rows of h further apart than 16 MiB
    assert L.mtpc_cp_loglik(C.byref(_head(workspace_bytes=16)), tg, out) == WS
    assert L.mtpc_cp_loglik(C.byref(_head(workspace=None)), tg, out) == NULL
    lay = binding.mtpc_sumlayers(0x6000, 4, 0)
    assert L.mtpc_btree_loglik(C.byref(_head(n=6)), C.byref(lay), tg, out) == UNSUP
    assert L.mtpc_hmm_loglik(C.byref(_head()), None, tg, out) == NULL
    bad = binding.mtpc_sumlayers(0x6000, 3, 0)
    assert L.mtpc_hmm_loglik(C.byref(_head()), C.byref(bad), tg, out) == SHAPE
    assert L.mtpc_cp_marginals(C.byref(_head()), tg, 9, out) == UNSUP
    assert L.mtpc_cp_sample(C.byref(_head()), 0, 1, 0, out, None, None, None) == SHAPE
    assert L.mtpc_cp_sample(C.byref(_head()), 2, 1, 0, None, None, None, None) == NULL
    assert L.mtpc_philox_uniforms(1, 1, 0, 0, 0, out, None) == SHAPE
    # verify: required pointers depend on the mode; nothing is launched on error
    assert L.mtpc_cp_verify(C.byref(_head()), out, tg, out, out, 0, 1, 0, None, tg) == NULL
    assert L.mtpc_cp_verify(C.byref(_head()), None, tg, out, out, 0, 1, 0, tg, tg) == NULL
    assert L.mtpc_cp_verify(C.byref(_head()), out, tg, None, out, 0, 1, 0, tg, tg) == NULL
    assert L.mtpc_cp_verify(C.byref(_head()), out, tg, out, out, 5, 1, 0, tg, tg) == UNSUP
    assert L.mtpc_cp_verify(C.byref(_head(workspace_bytes=16)), None, tg, None, out, 1, 0, 0, tg, tg) == WS
    assert L.mtpc_hmm_verify(C.byref(_head()), None, out, tg, out, out, 0, 1, 0, tg, tg) == NULL
    # scores from a table
    assert L.mtpc_cp_table_scores(C.byref(_head()), None, tg, 1, 0, out) == NULL
    assert L.mtpc_cp_table_scores(C.byref(_head()), out, None, 1, 0, out) == NULL
    assert L.mtpc_cp_table_scores(C.byref(_head()), out, tg, 0, 0, out) == SHAPE
    assert L.mtpc_cp_table_scores(C.byref(_head()), out, tg, 1, 2, out) == UNSUP
    assert L.mtpc_cp_table_scores(C.byref(_head(workspace_bytes=16)), out, tg, 1, 0, out) == WS
    assert L.mtpc_btree_table_scores(C.byref(_head()), None, out, tg, 1, 0, out) == NULL
    # several windows per position in one pass
    assert L.mtpc_cp_window_scores(C.byref(_head()), None, 1, None, 0, 0, out) == NULL
    assert L.mtpc_cp_window_scores(C.byref(_head()), tg, 1, None, 2, 0, out) == NULL
    assert L.mtpc_cp_window_scores(C.byref(_head()), tg, 0, None, 0, 0, out) == SHAPE
    assert L.mtpc_cp_window_scores(C.byref(_head()), tg, 1, tg, -1, 0, out) == SHAPE
    assert L.mtpc_cp_window_scores(C.byref(_head()), tg, 1, None, 0, 3, out) == UNSUP
    assert L.mtpc_cp_window_scores(C.byref(_head(workspace_bytes=16)), tg, 1, tg, 1, 1, out) == WS
    assert L.mtpc_hmm_window_scores(C.byref(_head()), None, tg, 1, None, 0, 0, out) == NULL
    # greedy draft and training step
    assert L.mtpc_cp_greedy_draft(C.byref(_head()), None, None, None, None) == NULL
    assert L.mtpc_cp_greedy_draft(C.byref(_head(workspace_bytes=16)), tg, None, None, None) == WS
    assert L.mtpc_cp_loss_backward(C.byref(_head()), tg, out, out, out, out, None) == NULL
    assert L.mtpc_cp_loss_backward(C.byref(_head()), tg, None, out, out, out, out) == NULL
    assert L.mtpc_cp_loss_backward(C.byref(_head(workspace_bytes=16)), tg, out, out, out, out, out) == WS
    assert L.mtpc_ff_loss_backward(C.byref(_head(r=2)), tg, out, out, out, out) == SHAPE
    assert L.mtpc_hmm_loss_backward(C.byref(_head()), C.byref(lay), tg, out, out, out, out, out, None, None) == NULL
    gappy = binding.mtpc_sumlayers(0x6000, 4, 13)         # per-position logits that are not dense
    assert L.mtpc_hmm_loss_backward(C.byref(_head()), C.byref(gappy), tg, out, out, out, out, out, out, None) == UNSUP
    ctx = binding.mtpc_sumlayers(None, 0, 0, 0x7000, 4 * 64)
    mixed = binding.mtpc_sumlayers(0x6000, 0, 0, 0x7000, 4 * 64)   # one R per step but a shared bias
    assert L.mtpc_hmm_loss_backward(C.byref(_head()), C.byref(mixed), tg, out, out, out, out, out, out, out) == UNSUP
    assert L.mtpc_hmm_loss_backward(C.byref(_head()), C.byref(ctx), tg, out, out, out, out, out, None, None) == NULL


def test_workspace_query():
    from paper_2511_11346_amd import binding
    L = binding.lib()
    hd = _head()
    small = L.mtpc_workspace_bytes(binding.CP, binding.OP_LOGLIK, C.byref(hd), None, 1, 0)
    assert small >= 4 * (hd.B * hd.r + hd.B * hd.n * hd.r)
    s4 = L.mtpc_workspace_bytes(binding.CP, binding.OP_SAMPLE, C.byref(hd), None, 4, 0)
    s8 = L.mtpc_workspace_bytes(binding.CP, binding.OP_SAMPLE, C.byref(hd), None, 8, 0)
    assert s8 > s4 > 0
    assert L.mtpc_workspace_bytes(9, 0, C.byref(hd), None, 1, 0) == 0
    assert L.mtpc_workspace_bytes(binding.CP, binding.OP_SAMPLE, C.byref(hd), None, 0, 0) == 0
    t1 = L.mtpc_workspace_bytes(binding.CP, binding.OP_TABLE, C.byref(hd), None, 1, 0)
    t16 = L.mtpc_workspace_bytes(binding.CP, binding.OP_TABLE, C.byref(hd), None, 16, 0)
    assert t16 >= 16 * 4 * hd.B * hd.n * hd.r and t16 > t1 == small
    assert L.mtpc_workspace_bytes(binding.CP, binding.OP_TABLE, C.byref(hd), None, 0, 0) == 0
    lay = binding.mtpc_sumlayers(0x6000, hd.r * hd.r, 0)
    hom = binding.mtpc_sumlayers(0x6000, 0, 0)
    a = L.mtpc_workspace_bytes(binding.HMM, binding.OP_LOGLIK, C.byref(hd), C.byref(lay), 1, 0)
    b = L.mtpc_workspace_bytes(binding.HMM, binding.OP_LOGLIK, C.byref(hd), C.byref(hom), 1, 0)
    assert a >= b > small


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and a C program that only
    includes it links against libmtpc.so and reads its status strings (no GPU call)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "abi.c"
    src.write_text(
        '#include "mtpc.h"\n#include <stdio.h>\n#include <string.h>\n'
        "int main(void) {\n"
        "  mtpc_head hd; memset(&hd, 0, sizeof hd);\n"
        "  if (mtpc_cp_loglik(&hd, 0, 0) == MTPC_OK) return 2;\n"          # rejected on the host
        "  if (mtpc_workspace_bytes(MTPC_CP, MTPC_OP_LOGLIK, &hd, 0, 1, 0) != 0) return 3;\n"
        '  printf("%s\\n", mtpc_status_string(MTPC_ERR_WORKSPACE));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "abi"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), LIB, "-Wl,-rpath," + os.path.dirname(LIB)], check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True)
    assert res.returncode == 0 and res.stdout.strip() != ""


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU fallback: without the built shared library every call raises."""
    from paper_2511_11346_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libmtpc.so"))
    with pytest.raises(binding.MtpcError, match="not found"):
        binding.lib()
    with pytest.raises(binding.MtpcError):
        binding.profile_unembed(None, None)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "ONE GPU" in res.stderr and res.stdout.strip() == ""
