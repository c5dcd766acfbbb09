"""Helpers of the GPU parity tests: upload seeded inputs, call the HIP library
through its binding, compare with the CPU oracle."""
import numpy as np
import torch

import mtpc_inputs as mi
from oracle import mtpc_oracle as oc
from oracle import speculative as sp

FP32_ABS = 1e-4      # log-likelihood tolerance for fp32 inputs
BF16_REL = 2e-3      # relative tolerance for bf16 inputs with fp32 accumulation
BOUNDARY = 1e-6      # uniforms closer than this to a CDF step are not compared


def to_dev(x, bits=None):
    if bits is not None:
        return torch.from_numpy(bits.copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def make_head(inp: mi.HeadInputs, layers=None):
    from paper_2511_11346_amd import Head
    bf = inp.dtype == "bf16"
    h = to_dev(inp.h, inp.h_bits if bf else None)
    W = to_dev(inp.W, inp.W_bits if bf else None)
    Wsum = None if inp.Wsum is None else to_dev(inp.Wsum, inp.Wsum_bits if bf else None)
    lay = inp.layers if layers is None else layers
    lay_t = None if lay is None or lay.size == 0 else to_dev(lay.astype(np.float32))
    R = None if inp.R is None else to_dev(inp.R, inp.R_bits if bf else None)
    return Head(inp.family, h, W, Wsum, lay_t, R=R)


def tol_check(got, want, dtype, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    both_nan = np.isnan(got) & np.isnan(want)
    both_ninf = np.isneginf(got) & np.isneginf(want)
    ok_special = both_nan | both_ninf
    assert np.array_equal(np.isnan(got), np.isnan(want)), what + ": NaN pattern differs"
    fin = ~ok_special
    err = np.abs(got[fin] - want[fin])
    if dtype == "f32":
        # also for windows of 64 tokens (|log q| up to 350, where an fp32 unit is 3e-5): the chains
        # keep their messages relative to the largest unit and sum the magnitude in double
        assert err.size == 0 or err.max() <= FP32_ABS, f"{what}: max abs err {err.max():.3e}"
    else:
        lim = BF16_REL * np.maximum(np.abs(want[fin]), 1e-2)
        assert err.size == 0 or np.all(err <= lim), f"{what}: max err {err.max():.3e}"
        # bf16 inputs are exact in fp32, so the fp32-accumulated result is in fact close
        assert err.size == 0 or err.max() <= 2e-3, f"{what}: max abs err {err.max():.3e}"
    return float(err.max()) if err.size else 0.0


def compare_drafts(g_drafts, g_lat, o_drafts, o_lat, margin):
    """Bit-exact outside the boundary set; returns (#boundary drafts, #mismatching boundary drafts)."""
    safe = margin >= BOUNDARY
    gd, gl = g_drafts.cpu().numpy(), (g_lat.cpu().numpy() if g_lat is not None else None)
    assert np.array_equal(gd[safe], o_drafts[safe]), "draft tokens differ away from CDF boundaries"
    if gl is not None and o_lat.shape[-1] > 0:
        assert np.array_equal(gl[safe], o_lat[safe]), "latents differ away from CDF boundaries"
    near = ~safe
    bad = int(np.any(gd[near] != o_drafts[near], axis=-1).sum()) if near.any() else 0
    return int(near.sum()), bad


def oracle_params(inp):
    lay = inp.layers
    if inp.R is not None:
        lay = oc.contextual_layer_logits(inp.h, inp.R, inp.layers)
    return oc._params(inp.family, inp.h, inp.W, inp.Wsum, lay)


def synthetic_verifier(inp, logphi, logw, loglayers, drafts, seed):
    """p[b,i] = (1-eps_b) q(. | x_<i) + eps_b noise, eps_b cycling through the batch."""
    B, n, r, v = logphi.shape
    noise = mi.verifier_noise(B, n, v, seed)
    eps = np.array([0.0, 0.03, 0.08, 0.15, 0.3, 1.0])[np.arange(B) % 6]
    p = noise.copy()
    for b in range(B):
        lay = None if loglayers is None else (loglayers[b] if loglayers.ndim == 4 else loglayers)
        for i in range(n):
            q = np.exp(sp.conditional_next(inp.family, logphi[b], None if logw is None else logw[b],
                                           lay, drafts[b], i))
            p[b, i] = (1 - eps[b]) * q + eps[b] * noise[b, i]
    return p / p.sum(axis=-1, keepdims=True)
