"""GPU parity of the operations on several windows per position and on the table of
normalised input units log phi[B][n][r][v]: scores of arbitrary windows from the table
(log-likelihood / prefix marginals without another pass over W) or from W in one pass, and
the two ways training-sized batches draw their tokens (Alg. 1): from the table when the
caller keeps it, else through buckets of (token, selected input unit)."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi
from oracle import mtpc_oracle as oc
from oracle import philox
from oracle import speculative as sp

from gpu_util import BOUNDARY, compare_drafts, make_head, oracle_params, tol_check

pytestmark = pytest.mark.gpu

CASES = [
    # family, dtype, B, d, n, r, v, contextual
    ("ff", "f32", 70, 64, 5, 1, 100, False),
    ("ff", "bf16", 9, 64, 3, 1, 320, False),
    ("cp", "bf16", 300, 128, 8, 16, 320, False),
    ("cp", "f32", 130, 64, 4, 5, 33, False),
    ("hmm", "f32", 65, 64, 6, 4, 130, False),
    ("hmm", "bf16", 140, 128, 8, 32, 320, True),
    ("btree", "bf16", 260, 64, 4, 16, 268, False),
    ("btree", "f32", 97, 64, 16, 8, 257, False),
    ("btree", "bf16", 33, 128, 8, 8, 100, True),
]


def windows(inp, T, seed):
    """T windows per position: uniform ids, some variables summed out, one invalid id."""
    B, n, v = inp.h.shape[0], inp.W.shape[0], inp.W.shape[2]
    rng = np.random.default_rng([seed, B, n, v])
    x = rng.integers(0, v, size=(B, T, n)).astype(np.int32)
    x[rng.random(x.shape) < 0.15] = -1
    x[0, 0, :] = -1                    # everything summed out: log 1 = 0
    if B > 1:
        x[1, T - 1, n - 1] = v         # invalid id: the outputs that observe it are NaN
    return x


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,ctx", CASES)
def test_table_scores_match_the_oracle(family, dtype, B, d, n, r, v, ctx):
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=900 + B + r, h_scale=1.0,
                         contextual=ctx)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    T = 3
    x = windows(inp, T, 17)
    xd = torch.from_numpy(x).cuda()
    want_P = np.stack([oc.prefix_marginals_from(family, logphi, logw, loglayers, x[:, t]) for t in range(T)], axis=1)
    want_L = np.stack([oc.joint(family, oc.evidence(logphi, x[:, t]), logw, loglayers) for t in range(T)], axis=1)

    # the table as the oracle computes it: only the sum units carry the dtype's tolerance
    tab = torch.from_numpy(logphi.astype(np.float32)).cuda()
    tol_check(head.table_scores(tab, xd, prefix=True).cpu().numpy(), want_P, dtype, "prefix scores, oracle table")
    got_L = head.table_scores(tab, xd).cpu().numpy()
    tol_check(got_L, want_L, dtype, "log-likelihoods, oracle table")
    assert abs(got_L[0, 0]) < 1e-5

    # the table a sampling call leaves (training-sized batches: written by the evidence kernel)
    table = torch.empty(B, n, r, v, dtype=torch.float32, device="cuda")
    head.sample(1, seed=3, want_prefix=False, logphi=table)
    tol_check(table.cpu().numpy(), logphi, dtype, "log phi table")
    tol_check(head.table_scores(table, xd, prefix=True).cpu().numpy(), want_P, dtype, "prefix scores, own table")
    tol_check(head.table_scores(table, xd).cpu().numpy(), want_L, dtype, "log-likelihoods, own table")
    # one window per position, 2-dim form; equals the fused evidence path to rounding
    one = head.table_scores(table, xd[:, 2].contiguous())
    ref = head.loglik(xd[:, 2].contiguous())
    fin = torch.isfinite(ref)
    assert torch.equal(torch.isnan(one), torch.isnan(ref))
    assert float((one[fin] - ref[fin]).abs().max()) < 2e-5


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,ctx", [c for c in CASES if c[2] > 64])
def test_draws_from_the_table_match_the_oracle(family, dtype, B, d, n, r, v, ctx):
    """Batches above 64 positions that keep the table draw their tokens from it."""
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=40 + B + n, h_scale=1.0,
                         contextual=ctx)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    S, seed, off = 2, 0xFEDCBA9876543210, 9
    u = philox.uniforms(B, S, n + oc.n_latents(family, n), seed, off)
    od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u, with_margin=True)
    table = torch.empty(B, n, r, v, dtype=torch.float32, device="cuda")
    gd, gl, gp = head.sample(S, seed=seed, offset=off, want_prefix=True, logphi=table)
    near, bad = compare_drafts(gd, gl, od, ol, margin)
    print(f"{family}: {near} of {margin.size} drafts within {BOUNDARY} of a CDF step, {bad} of those differ")
    assert near <= max(4, margin.size // 50)
    gdn = gd.cpu().numpy()
    assert gdn.min() >= 0 and gdn.max() < v
    for s in range(S):
        ps = oc.prefix_marginals_from(family, logphi, logw, loglayers, gdn[:, s])
        tol_check(gp[:, s].cpu().numpy(), ps, dtype, "draft prefix scores")

    # without the table the same draws go through the buckets
    gd3, gl3, gp3 = head.sample(S, seed=seed, offset=off, want_prefix=True)
    near3, _ = compare_drafts(gd3, gl3, od, ol, margin)
    assert near3 == near
    for s in range(S):
        ps = oc.prefix_marginals_from(family, logphi, logw, loglayers, gd3.cpu().numpy()[:, s])
        tol_check(gp3[:, s].cpu().numpy(), ps, dtype, "draft prefix scores (bucket path)")

    # greedy draft through both paths
    want_d, want_l, gap = sp.greedy_draft(family, logphi, logw, loglayers)
    safe = gap >= 1e-6
    for tab in (table, None):
        g2, l2, p2 = head.greedy_draft(want_prefix=True, logphi=tab)
        assert np.array_equal(g2.cpu().numpy()[safe], want_d[safe])
        if l2 is not None and want_l.shape[1]:
            assert np.array_equal(l2.cpu().numpy()[safe], want_l[safe])
        tol_check(p2.cpu().numpy(), oc.prefix_marginals_from(family, logphi, logw, loglayers, g2.cpu().numpy()),
                  dtype, "scores of the greedy draft")


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,ctx", CASES)
def test_window_scores_match_the_oracle(family, dtype, B, d, n, r, v, ctx):
    """Two sets of windows per position scored in one unembedding pass."""
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=700 + B + r, h_scale=1.0,
                         contextual=ctx)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    x = windows(inp, 3, 23)
    xa = torch.from_numpy(np.ascontiguousarray(x[:, :2])).cuda()
    xb = torch.from_numpy(np.ascontiguousarray(x[:, 2:])).cuda()
    want_P = np.stack([oc.prefix_marginals_from(family, logphi, logw, loglayers, x[:, t]) for t in range(3)], axis=1)
    want_L = np.stack([oc.joint(family, oc.evidence(logphi, x[:, t]), logw, loglayers) for t in range(3)], axis=1)
    tol_check(head.window_scores(xa, xb, prefix=True).cpu().numpy(), want_P, dtype, "prefix scores of two window sets")
    tol_check(head.window_scores(xa, xb).cpu().numpy(), want_L, dtype, "log-likelihoods of two window sets")
    tol_check(head.window_scores(xb).cpu().numpy(), want_L[:, 2:], dtype, "log-likelihoods of one window set")
    # one window per position: the very numbers of the loglik call
    assert torch.equal(head.window_scores(xb)[:, 0].nan_to_num(7.0), head.loglik(xb[:, 0].contiguous()).nan_to_num(7.0))


def test_rows_of_h_spread_over_more_than_4_gib():
    """h as a strided view whose rows lie 16 MiB apart: the gathered draw kernel addresses h
    through one 32-bit resource and must not be used; the in-kernel draws take over."""
    from paper_2511_11346_amd import Head
    B, d, n, r, v = 300, 64, 4, 8, 268
    inp = mi.make_inputs("hmm", B=B, d=d, n=n, r=r, v=v, dtype="bf16", seed=77, h_scale=1.0)
    ld = 1 << 23                                               # elements: 16 MiB per row, 4.7 GiB in all
    big = torch.zeros(B, ld, dtype=torch.bfloat16, device="cuda")
    big[:, :d] = torch.from_numpy(inp.h_bits.copy()).view(torch.bfloat16).cuda()
    as_dev = lambda bits: torch.from_numpy(bits.copy()).view(torch.bfloat16).cuda()
    head = Head("hmm", big[:, :d], as_dev(inp.W_bits), as_dev(inp.Wsum_bits),
                torch.from_numpy(inp.layers.astype(np.float32)).cuda())
    logphi, logw, loglayers = oracle_params(inp)
    S, seed = 2, 31
    u = philox.uniforms(B, S, n + oc.n_latents("hmm", n), seed, 0)
    od, ol, margin = oc.sample_from("hmm", logphi, logw, loglayers, u, with_margin=True)
    gd, gl, gp = head.sample(S, seed=seed, want_prefix=True)
    near, _ = compare_drafts(gd, gl, od, ol, margin)
    assert near <= max(4, margin.size // 50)
    for s in range(S):
        ps = oc.prefix_marginals_from("hmm", logphi, logw, loglayers, gd.cpu().numpy()[:, s])
        tol_check(gp[:, s].cpu().numpy(), ps, "bf16", "draft prefix scores")
    tg = torch.from_numpy(inp.targets).cuda()
    want = oc.joint("hmm", oc.evidence(logphi, inp.targets), logw, loglayers)
    tol_check(head.loglik(tg).cpu().numpy(), want, "bf16", "loglik")


@pytest.mark.parametrize("family,B,n,r,v,flat", [
    ("cp", 300, 4, 8, 100, True),        # greedy with a flat mixture: every draft in bucket 0
    ("hmm", 70, 3, 128, 64, False),      # far more buckets than rows: most are empty
    ("btree", 513, 4, 2, 320, False),    # two units: buckets of a few hundred rows, ragged last tiles
])
def test_bucket_extremes(family, B, n, r, v, flat):
    inp = mi.make_inputs(family, B=B, d=64, n=n, r=r, v=v, dtype="f32", seed=5 + B, h_scale=1.0)
    if flat:
        inp.Wsum[...] = 0.0
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    S, seed = 2, 99
    u = philox.uniforms(B, S, n + oc.n_latents(family, n), seed, 0)
    od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u, with_margin=True)
    gd, gl, _ = head.sample(S, seed=seed)
    near, _ = compare_drafts(gd, gl, od, ol, margin)
    assert near <= max(4, margin.size // 50)
    want_d, want_l, gap = sp.greedy_draft(family, logphi, logw, loglayers)
    g2, l2, _ = head.greedy_draft()
    if flat:
        # the mixture is an exact tie (first index wins on both sides): only the token decisions count
        assert np.all(l2.cpu().numpy() == 0) and np.all(want_l == 0)
        top2 = np.sort(np.exp(logphi[:, :, 0, :]), axis=-1)[..., -2:]
        safe = (top2[..., 1] - top2[..., 0]).min(axis=1) >= 1e-6
        assert safe.sum() >= B // 2
    else:
        safe = gap >= 1e-6
    assert np.array_equal(g2.cpu().numpy()[safe], want_d[safe])


@pytest.mark.parametrize("family,B,n,r,v", [
    ("cp", 4950, 8, 33, 300),        # 264 buckets whose sizes follow the mixture weights: from a few rows to several tiles
    ("hmm", 7200, 6, 48, 200),       # 288 buckets of about 150 rows, the 256-row vocabulary tile
    ("btree", 6000, 8, 40, 100),     # 320 buckets, the 128-row vocabulary tile
])
def test_gathered_draws_on_the_wide_tiles(family, B, n, r, v):
    """Shapes for which the bucketed draws take their 192-row tiles (more than 256 buckets of 112 to 172
    rows on average: one wide tile per bucket instead of two of 128 rows, a round over the CUs less):
    drafts and latents of sampled rows against the oracle, the greedy draft too."""
    inp = mi.make_inputs(family, B=B, d=64, n=n, r=r, v=v, dtype="bf16", seed=40 + r, h_scale=1.0)
    head = make_head(inp)
    rng = np.random.default_rng(B)
    rows = np.unique(np.concatenate([np.arange(8), np.arange(B - 8, B), rng.integers(0, B, 80)]))
    logphi, logw, loglayers = oc._params(family, inp.h[rows], inp.W, inp.Wsum, inp.layers)
    S, seed = 1, 7
    u = philox.uniforms(B, S, n + oc.n_latents(family, n), seed, 0)
    od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u[rows], with_margin=True)
    gd, gl, _ = head.sample(S, seed=seed)
    near, _ = compare_drafts(gd[rows], gl[rows] if gl is not None else None, od, ol, margin)
    assert near <= max(4, margin.size // 50)
    assert int(gd.min()) >= 0 and int(gd.max()) < v
    want_d, want_l, gap = sp.greedy_draft(family, logphi, logw, loglayers)
    g2, l2, _ = head.greedy_draft()
    safe = gap >= 1e-6
    assert safe.sum() >= len(rows) // 2
    assert np.array_equal(g2.cpu().numpy()[rows][safe], want_d[safe])
    # the same draws again: the order of the rows inside a bucket (atomics) changes nothing
    gd2, _, _ = head.sample(S, seed=seed)
    assert torch.equal(gd2, gd)


@pytest.mark.parametrize("family,dtype,B,S,d,n,r,v,ctx", [
    ("cp", "bf16", 1, 1, 4096, 16, 32, 320, False),     # batch-1 decoding at the full head width
    ("cp", "f32", 2, 2, 96, 4, 8, 33, False),           # exactly 2 B S = r
    ("hmm", "bf16", 3, 2, 160, 6, 16, 257, True),       # d with a ragged last group of chunks
    ("btree", "f32", 1, 3, 64, 8, 6, 100, False),
    ("btree", "f32", 4, 1, 2080, 4, 128, 40, False),    # d beyond one register-resident piece of h
])
def test_a_handful_of_drafts_without_scores(family, dtype, B, S, d, n, r, v, ctx):
    """With 2 B S <= r and no scores asked for, only the input unit each token is drawn from
    is evaluated (dot products instead of the pass over W): same draws, same greedy draft."""
    assert 2 * B * S <= r
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=17 + d + n, h_scale=1.0,
                         contextual=ctx)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    seed, off = 0x0123456789ABCDEF, 4
    near_sum = 0
    for k in range(4):                                   # few tokens a call: several calls
        u = philox.uniforms(B, S, n + oc.n_latents(family, n), seed, off + k)
        od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u, with_margin=True)
        gd, gl, gp = head.sample(S, seed=seed, offset=off + k)
        assert gp is None
        gdn = gd.cpu().numpy()
        assert gdn.min() >= 0 and gdn.max() < v
        near, _ = compare_drafts(gd, gl, od, ol, margin)
        near_sum += near
        # the pass over all of W (scores asked for) draws the same tokens
        gd2, gl2, _ = head.sample(S, seed=seed, offset=off + k, want_prefix=True)
        same = (gd2 == gd).all(dim=-1).cpu().numpy()
        assert np.all(same | (margin.reshape(same.shape) < BOUNDARY))
    assert near_sum <= 2
    if 2 * B <= r:
        want_d, want_l, gap = sp.greedy_draft(family, logphi, logw, loglayers)
        safe = gap >= 1e-6
        g2, l2, _ = head.greedy_draft()
        assert np.array_equal(g2.cpu().numpy()[safe], want_d[safe])
        if l2 is not None and want_l.shape[1]:
            assert np.array_equal(l2.cpu().numpy()[safe], want_l[safe])


@pytest.mark.parametrize("family,dtype,B,d,n,r,v", [
    ("cp", "bf16", 64, 4096, 16, 32, 320), ("cp", "bf16", 1, 256, 4, 8, 320), ("hmm", "f32", 33, 64, 5, 6, 130),
    ("btree", "bf16", 8, 128, 8, 16, 268), ("ff", "f32", 20, 96, 3, 1, 100),
    # more than 64 positions: the 256-position tiles, 64-byte stages
    ("cp", "bf16", 300, 128, 4, 5, 320), ("btree", "f32", 130, 64, 8, 16, 100), ("hmm", "bf16", 513, 96, 3, 4, 200),
])
def test_stage_major_copy_of_W_gives_the_same_bits(family, dtype, B, d, n, r, v):
    """Calls that read the stage-major copy of W (mtpc_pack_weights) instead of its rows: same products
    in the same order, so every output is bit-identical - drafts, scores, the table of input units,
    likelihoods, univariate marginals, the training step.  Up to 64 positions the copy has 128-byte
    stages, above 64-byte ones; a copy with the other stage size is ignored."""
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=60 + n + r, h_scale=1.0)
    plain, packed, other = make_head(inp), make_head(inp), make_head(inp)
    packed.pack_W()
    sb = 128 if B <= 64 else 64
    assert packed.W_stage_bytes == sb
    # the copy itself: [slab][stage][row][sb bytes]
    es = 2 if dtype == "bf16" else 4
    stages = d * es // sb
    want = plain.W.view(torch.uint8).view(n * r, v, stages, sb).permute(0, 2, 1, 3).contiguous()
    assert torch.equal(packed.W_stage_major.view(torch.uint8).view(n * r, stages, v, sb), want)
    tg = torch.from_numpy(inp.targets).cuda()
    if (d * es) % 128 == 0 or sb == 128:
        other.pack_W(stage_bytes=192 - sb)      # the other size: made, handed over, not read
        assert torch.equal(plain.loglik(tg), other.loglik(tg))
    if B > 64:
        coef = torch.full((B, n), 1.0 / B, device="cuda")
        ga, gb = plain.loss_backward(tg, coef), packed.loss_backward(tg, coef)
        assert all(torch.equal(ga[k], gb[k]) for k in ga if ga[k] is not None)
    assert torch.equal(plain.loglik(tg), packed.loglik(tg))
    assert torch.equal(plain.prefix_marginals(tg), packed.prefix_marginals(tg))
    assert torch.equal(plain.univariate_marginals(), packed.univariate_marginals())
    ta, tb = (torch.empty(B, n, r, v, dtype=torch.float32, device="cuda") for _ in range(2))
    a = plain.sample(2, seed=3, offset=1, want_prefix=True, logphi=ta)
    b = packed.sample(2, seed=3, offset=1, want_prefix=True, logphi=tb)
    assert all(torch.equal(x, y) for x, y in zip(a, b)) and torch.equal(ta, tb)
    assert torch.equal(plain.greedy_draft()[0], packed.greedy_draft()[0])
    # drafts alone: a large batch draws each token from its one slab, gathered (also from the copy)
    c = plain.sample(2, seed=4, want_prefix=False)
    e = packed.sample(2, seed=4, want_prefix=False)
    assert torch.equal(c[0], e[0]) and (c[1] is None or torch.equal(c[1], e[1]))
