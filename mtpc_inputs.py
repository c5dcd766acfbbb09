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

import os
from concurrent.futures import ThreadPoolExecutor
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
    R: Optional[np.ndarray] = None  # [L, r, r, d]: sum layers computed from h (then `layers` is the bias)
    R_bits: Optional[np.ndarray] = None
    meta: dict = field(default_factory=dict)


_CHUNK = 1 << 22


def _gauss(seed, tensor_id, shape, scale, bf16):
    """N(0, scale^2) of the given shape, drawn chunk by chunk from independent
    generators seeded (seed, tensor_id, chunk) so that the values do not depend on
    the number of worker threads.  Returns (fp32 values, bf16 bit patterns or
    None); with ``bf16`` the fp32 values are the rounded ones."""
    total = int(np.prod(shape))
    vals = np.empty(total, dtype=np.float32)
    bits = np.empty(total, dtype=np.uint16) if bf16 else None

    def work(c):
        lo, hi = c * _CHUNK, min(total, (c + 1) * _CHUNK)
        g = np.random.default_rng([seed, tensor_id, c])
        a = g.standard_normal(size=hi - lo, dtype=np.float32)
        a *= np.float32(scale)
        if bf16:
            b = f32_to_bf16_bits(a)
            bits[lo:hi] = b
            vals[lo:hi] = bf16_bits_to_f32(b)
        else:
            vals[lo:hi] = a

    nchunk = (total + _CHUNK - 1) // _CHUNK
    if nchunk <= 1:
        for c in range(nchunk):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(work, range(nchunk)))
    return vals.reshape(shape), (bits.reshape(shape) if bf16 else None)


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
                targets: str = "uniform", logit_gain: float = 1.0,
                contextual: bool = False) -> HeadInputs:
    """Draw one batch.

    h ~ N(0, h_scale^2) (default 1, or 1/sqrt(d) for bf16 workloads as the configs
    state), W, Wsum ~ N(0, 1/d) times ``logit_gain``, static layer logits ~ N(0, 1).
    ``layer_count`` overrides the number of r x r layers (1 = homogeneous HMM).
    ``contextual`` adds R [L,r,r,d] ~ N(0, 1/d): the layer logits are then R h + layers.
    """
    assert family in FAMILIES
    if family == "ff":
        assert r == 1
    rng = np.random.default_rng(seed)
    if h_scale is None:
        h_scale = 1.0 if dtype == "f32" else 1.0 / np.sqrt(d)
    if w_scale is None:
        w_scale = 1.0 / np.sqrt(d)
    if dtype not in ("f32", "bf16"):
        raise ValueError(dtype)
    bf = dtype == "bf16"
    h, h_bits = _gauss(seed, 1, (B, d), h_scale, bf)
    W, W_bits = _gauss(seed, 2, (n, r, v, d), w_scale * logit_gain, bf)
    Wsum, Wsum_bits = (None, None) if family == "ff" else _gauss(seed, 3, (r, d), w_scale * logit_gain, bf)
    layers = None
    if family == "hmm":
        L = (n - 1) if layer_count is None else layer_count
        layers, _ = _gauss(seed, 4, (L, r, r), 1.0, False)
    elif family == "btree":
        L = (n - 2) if layer_count is None else layer_count
        layers, _ = _gauss(seed, 4, (L, r, r), 1.0, False)
    if targets == "uniform":                  # every id of the vocabulary, also those beyond the bytes
        tg = rng.integers(0, v, size=(B, n), dtype=np.int32)
    elif targets == "biased":
        tg = biased_byte_targets(rng, B, n)
    else:
        raise ValueError(targets)
    R = R_bits = None
    if contextual and layers is not None:
        R, R_bits = _gauss(seed, 5, (layers.shape[0], r, r, d), w_scale * logit_gain, bf)
    return HeadInputs(family, dtype, B, d, n, r, v, h, W, Wsum, layers, tg,
                      h_bits=h_bits, W_bits=W_bits, Wsum_bits=Wsum_bits, R=R, R_bits=R_bits)


# --------------------------------------------------------------------------
# the five named workloads
# --------------------------------------------------------------------------
def config1(seed: int = 1001) -> HeadInputs:
    """CP, fp32, B=64, d=256, n=4, r=8, v=256; h~N(0,1); targets uniform bytes."""
    return make_inputs("cp", B=64, d=256, n=4, r=8, v=256, dtype="f32", seed=seed,
                       h_scale=1.0, targets="uniform")


def config2(r: int, B: int = 8192, seed: int = 1002, targets: str = "biased") -> HeadInputs:
    """FF (r=1) or CP (r=16), bf16, d=4096, n=8, v=320, biased byte targets."""
    fam = "ff" if r == 1 else "cp"
    return make_inputs(fam, B=B, d=4096, n=8, r=r, v=320, dtype="bf16", seed=seed,
                       targets=targets)


def config3(B: int = 8192, seed: int = 1003, targets: str = "biased") -> HeadInputs:
    """HMM, bf16, d=4096, n=8, r=32, v=320, one shared static 32x32 transition."""
    return make_inputs("hmm", B=B, d=4096, n=8, r=32, v=320, dtype="bf16", seed=seed,
                       targets=targets, layer_count=1)


def config3_contextual(B: int = 8192, seed: int = 1013) -> HeadInputs:
    """The HMM variant the paper trains (App. HMM setup): contextual, inhomogeneous -
    7 transition layers whose logits are R[l] h + bias[l]; bf16, d=4096, n=8, r=32, v=320."""
    return make_inputs("hmm", B=B, d=4096, n=8, r=32, v=320, dtype="bf16", seed=seed,
                       targets="biased", contextual=True)


def config_llama_byte(family: str = "cp", n: int = 8, B: int = 2048, seed: int = 1020) -> HeadInputs:
    """Second model shape of the paper (Tab. model_specs): Llama-3.2-3B-Byte head in
    fp32, d=3072, v=268 (not a multiple of 32), r=32; B = one 2048-byte context."""
    return make_inputs(family, B=B, d=3072, n=n, r=32, v=268, dtype="f32", seed=seed,
                       h_scale=1.0 / np.sqrt(3072), targets="biased")


def config4(B: int = 4096, seed: int = 1004, targets: str = "biased") -> HeadInputs:
    """Binary tree, bf16, d=3072, n=16, r=64, v=320, 14 static 64x64 sum layers."""
    return make_inputs("btree", B=B, d=3072, n=16, r=64, v=320, dtype="bf16", seed=seed,
                       targets=targets)


def config5(B: int = 64, seed: int = 1005, targets: str = "biased") -> HeadInputs:
    """Decode-shaped CP, bf16, r=32, d=4096, n=16, v=320, B in {1, 8, 64}."""
    return make_inputs("cp", B=B, d=4096, n=16, r=32, v=320, dtype="bf16", seed=seed,
                       targets=targets)


def verifier_noise(B: int, n: int, v: int, seed: int, peak: float = 3.0) -> np.ndarray:
    """Random categorical tables [B, n+1, v] (float64, rows sum to 1): softmax of
    peak * N(0,1) logits.  Raw material for synthetic verifier distributions of
    the speculative-decoding step; the tests and the bench mix it with the draft
    model's own conditionals to get a spread of acceptance lengths."""
    g = np.random.default_rng([seed, 77]).standard_normal((B, n + 1, v)) * peak
    g -= g.max(axis=-1, keepdims=True)
    p = np.exp(g)
    return p / p.sum(axis=-1, keepdims=True)
