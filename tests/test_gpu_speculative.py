"""GPU parity of the verification step (Alg. 2 from the acceptance loop on) and of
the input-unit table the sampler keeps for it.

The verifier distributions are synthetic: along each draft they are a mixture of
the draft model's own conditional (from the oracle) and random tables, with a
mixing weight that varies over the batch so that every acceptance length occurs.
Decisions are integers taken from floating-point comparisons; rows whose oracle
margin (distance of alpha from p/q, of the final uniform from a CDF step) is
below DECISION are counted and reported, all others must agree exactly."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi
from oracle import mtpc_oracle as oc
from oracle import philox
from oracle import speculative as sp

from gpu_util import make_head, oracle_params, synthetic_verifier, tol_check

pytestmark = pytest.mark.gpu

DECISION = 2e-5     # fp32 evaluation of ratios and partial sums of <= 320 terms


CASES = [
    # family, dtype, B, d, n, r, v, contextual
    ("ff", "f32", 21, 64, 4, 1, 268, False),
    ("cp", "bf16", 40, 256, 8, 16, 320, False),
    ("cp", "f32", 17, 64, 1, 5, 33, False),
    ("hmm", "f32", 33, 128, 8, 8, 268, False),
    ("hmm", "bf16", 61, 256, 16, 32, 320, True),
    ("btree", "bf16", 40, 256, 8, 16, 320, False),
    ("btree", "f32", 19, 64, 2, 3, 40, False),
    ("btree", "f32", 47, 64, 16, 128, 64, False),
    ("btree", "bf16", 12, 128, 4, 8, 100, True),
]


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,ctx", CASES)
def test_verify_matches_oracle(family, dtype, B, d, n, r, v, ctx):
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=300 + n + r, h_scale=1.0,
                         contextual=ctx)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    nl = oc.n_latents(family, n)

    # --- the sampler's table of input units
    table = torch.empty(B, n, r, v, dtype=torch.float32, device="cuda")
    gd, _, gp = head.sample(1, seed=11, want_prefix=True, logphi=table)
    tol_check(table.cpu().numpy(), logphi, dtype, "log phi table")

    # --- verification on inputs built by the oracle alone
    od, _ = oc.sample_from(family, logphi, logw, loglayers, philox.uniforms(B, 1, n + nl, 11, 0))
    drafts = od[:, 0].astype(np.int32)
    P = oc.prefix_marginals_from(family, logphi, logw, loglayers, drafts)
    p = synthetic_verifier(inp, logphi, logw, loglayers, drafts, seed=5)
    u = philox.verify_uniforms(B, n + 1, 12, 3)
    best = p.argmax(axis=-1)
    greedy_drafts = best[:, :n].astype(np.int32)             # argmax chain, broken at position b % (n+1)
    for b in range(B):
        k = b % (n + 1)
        if k < n:
            greedy_drafts[b, k] = (greedy_drafts[b, k] + 1 + b) % v
    for mode, dr in (("sampling", drafts), ("greedy", greedy_drafts)):
        want_acc, want_tok, margin = sp.speculative_verify(family, logphi, logw, loglayers, dr, p, u, mode=mode)
        acc, tok = head.verify(torch.from_numpy(dr).cuda(), torch.from_numpy(p.astype(np.float32)).cuda(),
                               prefix_logq=torch.from_numpy(P.astype(np.float32)).cuda(),
                               logphi=torch.from_numpy(logphi.astype(np.float32)).cuda(),
                               seed=12, offset=3, mode=mode)
        acc, tok = acc.cpu().numpy(), tok.cpu().numpy()
        safe = margin >= DECISION
        assert np.array_equal(acc[safe], want_acc[safe]), (mode, acc, want_acc)
        assert np.array_equal(tok[safe], want_tok[safe]), (mode, tok, want_tok)
        assert np.all((acc >= 0) & (acc <= n) & (tok >= 0) & (tok < v))
        near = int((~safe).sum())
        bad = int(((acc != want_acc) | (tok != want_tok))[~safe].sum())
        print(f"{family} {dtype} n={n} r={r} {mode}: accepted histogram {np.bincount(want_acc, minlength=n + 1)}, "
              f"{near} of {B} rows within {DECISION} of a decision boundary, {bad} of those differ")
        if B >= 15:
            assert len(np.unique(want_acc)) >= 2

    # --- end to end: the library's own draft, scores and table (same seed as the
    # oracle's draft, so the drafts coincide except at CDF boundaries)
    gdn = gd[:, 0].contiguous()
    same = np.all(gdn.cpu().numpy() == drafts, axis=1)
    acc2, tok2 = head.verify(gdn, torch.from_numpy(p.astype(np.float32)).cuda(), prefix_logq=gp[:, 0].contiguous(),
                             logphi=table, seed=12, offset=3)
    w_acc, w_tok, margin2 = sp.speculative_verify(family, logphi, logw, loglayers, drafts, p, u)
    lim = 4e-3 if dtype == "bf16" else 2e-4          # decisions now also see the tolerance of scores and table
    safe = same & (margin2 >= lim)
    assert np.array_equal(acc2.cpu().numpy()[safe], w_acc[safe])
    assert np.array_equal(tok2.cpu().numpy()[safe], w_tok[safe])
    assert safe.sum() >= B // 2


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,ctx", CASES)
def test_greedy_draft_matches_oracle(family, dtype, B, d, n, r, v, ctx):
    """The argmax traversal (Sec. 3.4): bit-exact for every position none of whose decisions
    has its two largest probabilities closer than 1e-6; its prefix scores to tolerance; and
    drafting greedily against a verifier equal to the draft accepts everything."""
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=500 + n + r, h_scale=1.0,
                         contextual=ctx)
    head = make_head(inp)
    logphi, logw, loglayers = oracle_params(inp)
    want_d, want_l, gap = sp.greedy_draft(family, logphi, logw, loglayers)
    gd, gl, gp = head.greedy_draft(want_prefix=True)
    safe = gap >= 1e-6
    assert np.array_equal(gd.cpu().numpy()[safe], want_d[safe])
    if gl is not None and want_l.shape[1]:
        assert np.array_equal(gl.cpu().numpy()[safe], want_l[safe])
    P = oc.prefix_marginals_from(family, logphi, logw, loglayers, gd.cpu().numpy())
    tol_check(gp.cpu().numpy(), P, dtype, "scores of the greedy draft")
    onehot = torch.zeros(B, n + 1, v, device="cuda")
    onehot[:, :n].scatter_(2, gd.long()[:, :, None], 1.0)
    onehot[:, n, 0] = 1.0
    acc, tok = head.verify(gd, onehot, mode="greedy")
    assert torch.all(acc == n) and torch.all(tok == 0)
    print(f"{family} {dtype}: {int((~safe).sum())} of {B} positions have a near-tie")
