"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element
by element on the same seeded inputs.  Sizes are small enough for the oracle to
finish in seconds yet span several tiles and ragged tails (B, v not multiples of
the tile, v below / above a 32-row block boundary)."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi
from oracle import mtpc_oracle as oc
from oracle import philox

from gpu_util import BOUNDARY, FP32_ABS, compare_drafts, make_head, tol_check

pytestmark = pytest.mark.gpu


def oracle_all(inp, layers=None):
    lay = inp.layers if layers is None else layers
    if lay is not None and lay.size == 0:
        lay = None
    return oc._params(inp.family, inp.h, inp.W, inp.Wsum, lay)


def test_philox_uniforms_match_the_oracle_bit_for_bit():
    from paper_2511_11346_amd import philox_uniforms
    for (B, S, slots, seed, off) in [(3, 2, 9, 0, 0), (5, 4, 37, (0xDEADBEEF << 32) | 0x1234, 77)]:
        g = philox_uniforms(B, S, slots, seed, off).cpu().numpy()
        o = philox.uniforms(B, S, slots, seed, off)
        assert np.array_equal(g.astype(np.float64), o)


def test_config1_cp_fp32_everything():
    """CP, fp32, B=64, d=256, n=4, r=8, v=256: loglik + both marginals + 4 drafts, seed 0."""
    inp = mi.config1()
    head = make_head(inp)
    logphi, logw, _ = oracle_all(inp)
    tg = torch.from_numpy(inp.targets).cuda()
    want = oc.joint("cp", oc.evidence(logphi, inp.targets), logw)
    tol_check(head.loglik(tg).cpu().numpy(), want, "f32", "loglik")
    P = oc.prefix_marginals_from("cp", logphi, logw, None, inp.targets)
    tol_check(head.prefix_marginals(tg).cpu().numpy(), P, "f32", "prefix")
    M = oc.univariate_marginals("cp", inp.h, inp.W, inp.Wsum, None)
    tol_check(head.univariate_marginals().cpu().numpy(), M, "f32", "univariate")
    u = philox.uniforms(64, 4, 4 + 1, seed=0)
    od, ol, margin = oc.sample_from("cp", logphi, logw, None, u, with_margin=True)
    gd, gl, gp = head.sample(4, seed=0, want_prefix=True)
    near, bad = compare_drafts(gd, gl, od, ol, margin)
    print(f"config1 drafts: {near} of {margin.size} within {BOUNDARY} of a CDF step, {bad} of those differ")
    assert near <= 8
    # prefix scores of the GPU's own drafts against the oracle on those drafts
    gdn = gd.cpu().numpy()
    for s in range(4):
        ps = oc.prefix_marginals_from("cp", logphi, logw, None, gdn[:, s])
        tol_check(gp[:, s].cpu().numpy(), ps, "f32", "draft prefix scores")


CASES = [
    # family, dtype, B, d, n, r, v
    ("ff", "f32", 70, 64, 5, 1, 100),
    ("ff", "bf16", 300, 96, 3, 1, 320),
    ("cp", "bf16", 300, 128, 4, 5, 268),
    ("cp", "f32", 33, 32, 2, 3, 7),
    ("hmm", "f32", 65, 64, 6, 4, 130),
    ("hmm", "bf16", 257, 64, 4, 32, 320),
    ("hmm", "bf16", 40, 64, 3, 70, 64),
    ("btree", "f32", 50, 64, 8, 3, 257),
    ("btree", "bf16", 260, 64, 4, 16, 320),
    ("btree", "bf16", 20, 32, 2, 4, 33),
    ("btree", "f32", 9, 32, 16, 66, 40),
]


@pytest.mark.parametrize("family,dtype,B,d,n,r,v", CASES)
def test_loglik_and_marginals(family, dtype, B, d, n, r, v):
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=B + n + r + v,
                         h_scale=1.0, logit_gain=1.0)
    tgt = np.array(inp.targets, copy=True)
    tgt %= v
    tgt[0, :] = -1                      # everything summed out: log 1 = 0
    tgt[1 % B, n // 2] = -1             # one variable summed out
    if B > 2:
        tgt[2, 0] = v                   # invalid id: NaN row
    head = make_head(inp)
    logphi, logw, loglayers = oracle_all(inp)
    tg = torch.from_numpy(tgt).cuda()
    want = oc.joint(family, oc.evidence(logphi, tgt), logw, loglayers)
    got = head.loglik(tg).cpu().numpy()
    tol_check(got, want, dtype, "loglik")
    assert abs(got[0]) < 1e-5
    P = oc.prefix_marginals_from(family, logphi, logw, loglayers, tgt)
    tol_check(head.prefix_marginals(tg).cpu().numpy(), P, dtype, "prefix")
    if B <= 70:
        lay = inp.layers if (inp.layers is not None and inp.layers.size) else None
        M = oc.univariate_marginals(family, inp.h, inp.W, inp.Wsum, lay)
        tol_check(head.univariate_marginals().cpu().numpy(), M, dtype, "univariate")
        tol_check(head.univariate_marginals(keep_table=False).cpu().numpy(), M, dtype, "univariate, mixed in registers")


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,S", [
    ("ff", "f32", 40, 64, 4, 1, 100, 3),
    ("cp", "bf16", 100, 64, 4, 5, 268, 2),
    ("hmm", "f32", 65, 64, 5, 4, 130, 3),
    ("hmm", "bf16", 30, 64, 3, 70, 320, 1),
    ("btree", "f32", 50, 64, 8, 3, 257, 2),
    ("btree", "bf16", 300, 64, 4, 16, 320, 1),
])
def test_sampling_matches_the_oracle(family, dtype, B, d, n, r, v, S):
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=7 * B + n, h_scale=1.0)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_all(inp)
    seed, off = 0x0123456789ABCDEF, 5
    u = philox.uniforms(B, S, n + oc.n_latents(family, n), seed, off)
    od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u, with_margin=True)
    gd, gl, gp = head.sample(S, seed=seed, offset=off, want_prefix=True)
    near, bad = compare_drafts(gd, gl, od, ol, margin)
    print(f"{family}: {near} of {margin.size} drafts within {BOUNDARY} of a CDF step, {bad} of those differ")
    assert near <= max(4, margin.size // 50)
    gdn = gd.cpu().numpy()
    assert gdn.min() >= 0 and gdn.max() < v
    for s in range(S):
        ps = oc.prefix_marginals_from(family, logphi, logw, loglayers, gdn[:, s])
        tol_check(gp[:, s].cpu().numpy(), ps, dtype, "draft prefix scores")
    # without the optional outputs the drafts are the same (large batches then draw inside the
    # fused kernel instead of from the table: same rule, so only boundary draws may differ)
    gd2, _, _ = head.sample(S, seed=seed, offset=off, want_latents=False, want_prefix=False)
    near2, _ = compare_drafts(gd2, None, od, ol, margin)
    assert near2 == near
    assert torch.equal(gd, gd2) or B > 64


def test_peaked_logits_and_forbidden_transitions():
    """Logits of std ~8 (sharp softmaxes) and -inf entries in the sum layers."""
    inp = mi.make_inputs("hmm", B=70, d=64, n=5, r=6, v=300, dtype="f32", seed=3, h_scale=1.0,
                         logit_gain=8.0)
    lay = np.array(inp.layers, copy=True)
    lay[:, :, 2] = -np.inf              # state 2 can never be entered
    lay[1, 3, :] = -np.inf
    lay[1, 3, 4] = 0.0                  # deterministic row
    head = make_head(inp, layers=lay)
    logphi, logw, loglayers = oracle_all(inp, layers=lay)
    tg = torch.from_numpy(inp.targets).cuda()
    want = oc.joint("hmm", oc.evidence(logphi, inp.targets), logw, loglayers)
    got = head.loglik(tg).cpu().numpy()
    assert np.all(np.isfinite(got))
    err = float(np.max(np.abs(got - want)))
    print(f"peaked logits: max abs err {err:.2e}")
    assert err <= FP32_ABS
    u = philox.uniforms(70, 2, 5 + 5, seed=11)
    od, ol, margin = oc.sample_from("hmm", logphi, logw, loglayers, u, with_margin=True)
    gd, gl, _ = head.sample(2, seed=11)
    compare_drafts(gd, gl, od, ol, margin)
    assert not np.any(gl.cpu().numpy()[:, :, 1:] == 2)


def test_identity_transitions_reduce_hmm_and_btree_to_cp():
    n, r = 4, 8
    inp = mi.make_inputs("cp", B=64, d=64, n=n, r=r, v=96, dtype="bf16", seed=21, h_scale=1.0)
    cp = make_head(inp)
    tg = torch.from_numpy(inp.targets).cuda()
    ref = cp.loglik(tg)
    eye = np.full((n - 1, r, r), -np.inf, dtype=np.float32)
    eye[:, np.arange(r), np.arange(r)] = 0.0
    inp.family = "hmm"
    assert torch.allclose(make_head(inp, layers=eye).loglik(tg), ref, atol=1e-5, rtol=0)
    inp.family = "btree"
    assert torch.allclose(make_head(inp, layers=eye[: n - 2]).loglik(tg), ref, atol=1e-5, rtol=0)


def test_contextual_and_homogeneous_layers():
    B, n, r = 37, 4, 5
    inp = mi.make_inputs("hmm", B=B, d=64, n=n, r=r, v=50, dtype="f32", seed=5, h_scale=1.0)
    rng = np.random.default_rng(0)
    ctx = rng.standard_normal((B, n - 1, r, r)).astype(np.float32)
    tg = torch.from_numpy(inp.targets).cuda()
    for lay in (ctx, inp.layers[:1]):
        head = make_head(inp, layers=lay)
        logphi, logw, loglayers = oracle_all(inp, layers=lay)
        want = oc.prefix_marginals_from("hmm", logphi, logw, loglayers, inp.targets)
        tol_check(head.prefix_marginals(tg).cpu().numpy(), want, "f32", "prefix")
    inp2 = mi.make_inputs("btree", B=B, d=64, n=8, r=r, v=50, dtype="f32", seed=6, h_scale=1.0)
    ctx2 = rng.standard_normal((B, 6, r, r)).astype(np.float32)
    head = make_head(inp2, layers=ctx2)
    logphi, logw, loglayers = oracle_all(inp2, layers=ctx2)
    tg2 = torch.from_numpy(inp2.targets).cuda()
    want = oc.prefix_marginals_from("btree", logphi, logw, loglayers, inp2.targets)
    tol_check(head.prefix_marginals(tg2).cpu().numpy(), want, "f32", "prefix ctx btree")
    u = philox.uniforms(B, 2, 8 + 7, seed=4)
    od, ol, margin = oc.sample_from("btree", logphi, logw, loglayers, u, with_margin=True)
    gd, gl, _ = head.sample(2, seed=4)
    compare_drafts(gd, gl, od, ol, margin)


def test_strided_hidden_states_and_determinism():
    inp = mi.make_inputs("cp", B=90, d=64, n=3, r=4, v=200, dtype="bf16", seed=9, h_scale=1.0)
    from paper_2511_11346_amd import Head
    head = make_head(inp)
    tg = torch.from_numpy(inp.targets).cuda()
    a = head.loglik(tg)
    wide = torch.zeros(90, 128, dtype=torch.bfloat16, device="cuda")
    wide[:, :64] = head.h
    h2 = Head("cp", wide[:, :64], head.W, head.Wsum)
    assert torch.equal(a, h2.loglik(tg))
    assert torch.equal(a, head.loglik(tg))


@pytest.mark.parametrize("family,dtype,B,d,n,r", [
    ("hmm", "f32", 70, 64, 4, 5), ("hmm", "bf16", 300, 128, 5, 32), ("btree", "bf16", 130, 64, 8, 16),
    ("btree", "f32", 33, 32, 4, 70), ("hmm", "bf16", 20, 64, 3, 8),
    # r a power of two and more than 64 positions: the dense-slab kernel, every unit size
    ("hmm", "f32", 100, 64, 3, 8), ("hmm", "bf16", 97, 64, 4, 16), ("hmm", "bf16", 130, 64, 3, 64),
    ("hmm", "f32", 70, 32, 2, 128),
])
def test_sum_layers_computed_from_the_hidden_state(family, dtype, B, d, n, r):
    """Sec. 3.3 / App. HMM setup: layer logits R[l,k] e_t + bias computed in the library."""
    from paper_2511_11346_amd import Head
    v = 64
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=3 * B + r, h_scale=1.0)
    L = n - 1 if family == "hmm" else n - 2
    Rv, Rbits = mi._gauss(77, 9, (L, r, r, d), 2.0 / np.sqrt(d), dtype == "bf16")
    bias = np.random.default_rng(1).standard_normal((L, r, r)).astype(np.float32)
    bias[:, 0, 1] = -np.inf                       # a forbidden transition through the bias
    from gpu_util import to_dev
    base = make_head(inp)
    head = Head(family, base.h, base.W, base.Wsum, to_dev(bias), R=to_dev(Rv, Rbits))
    lay = oc.contextual_layer_logits(inp.h, Rv, bias)
    logphi, logw, loglayers = oc._params(family, inp.h, inp.W, inp.Wsum, lay)
    tg = torch.from_numpy(inp.targets).cuda()
    want = oc.prefix_marginals_from(family, logphi, logw, loglayers, inp.targets)
    tol_check(head.prefix_marginals(tg).cpu().numpy(), want, dtype, "prefix, layers from h")
    tol_check(head.loglik(tg).cpu().numpy(), want[:, -1], dtype, "loglik, layers from h")
    S = 2
    u = philox.uniforms(B, S, n + oc.n_latents(family, n), seed=21)
    od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u, with_margin=True)
    gd, gl, gp = head.sample(S, seed=21, want_prefix=True)
    near, bad = compare_drafts(gd, gl, od, ol, margin)
    assert near <= max(4, margin.size // 25)
    gdn = gd.cpu().numpy()
    for s in range(S):
        ps = oc.prefix_marginals_from(family, logphi, logw, loglayers, gdn[:, s])
        tol_check(gp[:, s].cpu().numpy(), ps, dtype, "draft scores, layers from h")
    if B <= 70:
        M = oc.univariate_marginals(family, inp.h, inp.W, inp.Wsum, lay)
        tol_check(head.univariate_marginals().cpu().numpy(), M, dtype, "univariate, layers from h")
        tol_check(head.univariate_marginals(keep_table=False).cpu().numpy(), M, dtype,
                  "univariate, layers from h, mixed in registers")
    # shared R and no bias: one tensor for all layers
    head2 = Head(family, base.h, base.W, base.Wsum, None, R=to_dev(Rv[:1], None if Rbits is None else Rbits[:1]))
    lay2 = oc.contextual_layer_logits(inp.h, np.repeat(Rv[:1], L, axis=0))
    _, _, ll2 = oc._params(family, inp.h, inp.W, inp.Wsum, lay2)
    tol_check(head2.loglik(tg).cpu().numpy(), oc.joint(family, oc.evidence(logphi, inp.targets), logw, ll2),
              dtype, "loglik, shared R")


@pytest.mark.parametrize("dtype,B,d,n,r,v", [
    ("f32", 300, 64, 8, 64, 40), ("bf16", 277, 64, 16, 32, 100), ("f32", 513, 32, 4, 16, 33),
    ("bf16", 1000, 32, 32, 16, 20), ("f32", 256, 32, 16, 64, 7),
    # the longest windows whose node values still fit the LDS of a CU (146 and 150 KB), and 64 tokens
    ("f32", 270, 32, 32, 64, 5), ("bf16", 260, 32, 64, 32, 3), ("f32", 257, 32, 64, 16, 9),
])
def test_tree_layers_shared_by_all_rows_with_16_32_64_units(dtype, B, d, n, r, v):
    """Batches of at least 256 rows of a tree whose layers are shared and whose r is 16, 32 or 64
    evaluate their sum layers as matrix products (16 rows per wave): ragged row counts, layers
    with forbidden and deterministic transitions, summed-out and invalid targets, one and two
    windows per position."""
    inp = mi.make_inputs("btree", B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=90 + n + r, h_scale=1.0)
    lay = np.array(inp.layers, copy=True)
    lay[:, :, 2] = -np.inf                      # unit 2 of every inner node can never be entered
    lay[1, 3, :] = -np.inf
    lay[1, 3, 5] = 0.0                          # a deterministic row
    tg = np.array(inp.targets, copy=True)
    rng = np.random.default_rng(5)
    tg[rng.random(tg.shape) < 0.1] = -1
    tg[7, n // 2] = v + 3                       # an id outside the vocabulary: NaN from there on
    tg[B - 1, 0] = -5
    head = make_head(inp, layers=lay)
    logphi, logw, loglayers = oracle_all(inp, layers=lay)
    want = oc.prefix_marginals_from("btree", logphi, logw, loglayers, tg)
    assert np.isnan(want[7, n // 2:]).all() and not np.isnan(want[7, :n // 2]).any()
    tgd = torch.from_numpy(tg).cuda()
    tol_check(head.prefix_marginals(tgd).cpu().numpy(), want, dtype, "prefix marginals")
    tol_check(head.loglik(tgd).cpu().numpy(), want[:, -1], dtype, "loglik")
    other = np.array(inp.targets[::-1], copy=True)
    both = head.window_scores(tgd.view(B, 1, n), torch.from_numpy(other).cuda().view(B, 1, n), prefix=True).cpu().numpy()
    tol_check(both[:, 0], want, dtype, "first window of two")
    tol_check(both[:, 1], oc.prefix_marginals_from("btree", logphi, logw, loglayers, other), dtype, "second window of two")
