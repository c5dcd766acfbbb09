"""Seeded synthetic inputs for the MtPC head (shapes of the paper's workloads).

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests/bench.  It holds no arithmetic of the method: it only draws random tensors
of the right shape and distribution and, for bf16 workloads, rounds them to bf16
once so that both sides see the very same bit patterns.

Shapes follow the head's parametrisation (Sec. 3.3): hidden state h [B, d],
unembedding tensor W [n, r, v, d], sum-unit matrix Wsum [r, d]; the static r x r
sum layers are the HMM transitions (n-1 of them, or one shared) and the binary
tree's inner nodes (n-2).  The hidden sizes, vocabulary and window lengths are the
ones of the two byte-level models the paper retrofits (Tab. model_specs); no item
of its evaluation data is used or reproduced - the values are i.i.d. Gaussian.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

FAMILIES = ("ff", "cp", "hmm", "btree")


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class HeadInputs:
    """One synthetic batch.  Float tensors are fp32 arrays; when ``dtype`` is
    "bf16" their values are exactly representable in bf16 and ``*_bits`` holds the
    uint16 patterns to upload."""
    family: str
    dtype: str                      # "f32" | "bf16"
    B: int
    d: int
    n: int
    r: int
    v: int
    h: np.ndarray                   # [B, d]
    W: np.ndarray                   # [n, r, v, d]
    Wsum: Optional[np.ndarray]      # [r, d] (None for ff)
    layers: Optional[np.ndarray]    # [L, r, r] pre-softmax logits (hmm: L=n-1 or 1; btree: L=n-2)
    targets: np.ndarray             # [B, n] int32
    h_bits: Optional[np.ndarray] = None
    W_bits: Optional[np.ndarray] = None
    Wsum_bits: Optional[np.ndarray] = None
    meta: dict = field(default_factory=dict)


def _gauss(rng, shape, scale):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(scale)
    return a


def biased_byte_targets(rng, B: int, n: int) -> np.ndarray:
    """Uniform bytes, with probability 0.2 replaced by a printable-ASCII byte
    (32..126): a crude stand-in for text-like byte statistics."""
    t = rng.integers(0, 256, size=(B, n), dtype=np.int32)
    asc = rng.integers(32, 127, size=(B, n), dtype=np.int32)
    pick = rng.random(size=(B, n)) < 0.2
    return np.where(pick, asc, t).astype(np.int32)


def make_inputs(family: str, *, B: int, d: int, n: int, r: int, v: int,
                dtype: str = "bf16", seed: int = 0, h_scale: Optional[float] = None,
                w_scale: Optional[float] = None, layer_count: Optional[int] = None,
                targets: str = "uniform", logit_gain: float = 1.0) -> HeadInputs:
    """Draw one batch.

    h ~ N(0, h_scale^2) (default 1, or 1/sqrt(d) for bf16 workloads as the configs
    state), W, Wsum ~ N(0, 1/d) times ``logit_gain``, static layer logits ~ N(0, 1).
    ``layer_count`` overrides the number of r x r layers (1 = homogeneous HMM).
    """
    assert family in FAMILIES
    if family == "ff":
        assert r == 1
    rng = np.random.default_rng(seed)
    if h_scale is None:
        h_scale = 1.0 if dtype == "f32" else 1.0 / np.sqrt(d)
    if w_scale is None:
        w_scale = 1.0 / np.sqrt(d)
    h = _gauss(rng, (B, d), h_scale)
    W = _gauss(rng, (n, r, v, d), w_scale * logit_gain)
    Wsum = None if family == "ff" else _gauss(rng, (r, d), w_scale * logit_gain)
    layers = None
    if family == "hmm":
        L = (n - 1) if layer_count is None else layer_count
        layers = _gauss(rng, (L, r, r), 1.0)
    elif family == "btree":
        L = (n - 2) if layer_count is None else layer_count
        layers = _gauss(rng, (L, r, r), 1.0)
    if targets == "uniform":
        tg = rng.integers(0, min(v, 256), size=(B, n), dtype=np.int32)
    elif targets == "biased":
        tg = biased_byte_targets(rng, B, n)
    else:
        raise ValueError(targets)
    out = HeadInputs(family, dtype, B, d, n, r, v, h, W, Wsum, layers, tg)
    if dtype == "bf16":
        out.h_bits = f32_to_bf16_bits(h)
        out.h = bf16_bits_to_f32(out.h_bits)
        out.W_bits = f32_to_bf16_bits(W)
        out.W = bf16_bits_to_f32(out.W_bits)
        if Wsum is not None:
            out.Wsum_bits = f32_to_bf16_bits(Wsum)
            out.Wsum = bf16_bits_to_f32(out.Wsum_bits)
    elif dtype != "f32":
        raise ValueError(dtype)
    return out


# --------------------------------------------------------------------------
# the five named workloads
# --------------------------------------------------------------------------
def config1(seed: int = 1001) -> HeadInputs:
    """CP, fp32, B=64, d=256, n=4, r=8, v=256; h~N(0,1); targets uniform bytes."""
    return make_inputs("cp", B=64, d=256, n=4, r=8, v=256, dtype="f32", seed=seed,
                       h_scale=1.0, targets="uniform")


def config2(r: int, B: int = 8192, seed: int = 1002) -> HeadInputs:
    """FF (r=1) or CP (r=16), bf16, d=4096, n=8, v=320, biased byte targets."""
    fam = "ff" if r == 1 else "cp"
    return make_inputs(fam, B=B, d=4096, n=8, r=r, v=320, dtype="bf16", seed=seed,
                       targets="biased")


def config3(B: int = 8192, seed: int = 1003) -> HeadInputs:
    """HMM, bf16, d=4096, n=8, r=32, v=320, one shared static 32x32 transition."""
    return make_inputs("hmm", B=B, d=4096, n=8, r=32, v=320, dtype="bf16", seed=seed,
                       targets="biased", layer_count=1)


def config4(B: int = 4096, seed: int = 1004) -> HeadInputs:
    """Binary tree, bf16, d=3072, n=16, r=64, v=320, 14 static 64x64 sum layers."""
    return make_inputs("btree", B=B, d=3072, n=16, r=64, v=320, dtype="bf16", seed=seed,
                       targets="biased")


def config5(B: int = 64, seed: int = 1005) -> HeadInputs:
    """Decode-shaped CP, bf16, r=32, d=4096, n=16, v=320, B in {1, 8, 64}."""
    return make_inputs("cp", B=B, d=4096, n=16, r=32, v=320, dtype="bf16", seed=seed,
                       targets="biased")
