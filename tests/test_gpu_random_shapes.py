"""A seeded sweep over legal shapes (every family, both dtypes, windows from 1 to 64,
1 to 128 units, ragged vocabularies and batches): every operation of the library against
the oracle on each.  The shapes are drawn once from a fixed seed, so the sweep is the
same on every run; the oracle's cost per case is bounded."""
import os

import numpy as np
import pytest
import torch

import mtpc_inputs as mi
from oracle import backward as bw
from oracle import mtpc_oracle as oc
from oracle import philox
from oracle import speculative as sp

from gpu_util import compare_drafts, make_head, synthetic_verifier, tol_check

pytestmark = pytest.mark.gpu


def draw_cases(count=24, seed=20251127):
    # (a longer sweep from another seed: MTPC_SWEEP_COUNT / MTPC_SWEEP_SEED in the environment)
    count = int(os.environ.get("MTPC_SWEEP_COUNT", count))
    seed = int(os.environ.get("MTPC_SWEEP_SEED", seed))
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        family = ["ff", "cp", "hmm", "btree"][rng.integers(0, 4)]
        n = int(rng.choice([2, 4, 8, 16, 32, 64] if family == "btree" else [1, 2, 3, 5, 8, 16, 33, 64]))
        r = 1 if family == "ff" else int(rng.choice([1, 2, 3, 7, 8, 16, 31, 32, 64, 100, 128]))
        v = int(rng.choice([1, 2, 5, 33, 64, 100, 129, 256, 257, 268, 319, 320]))
        d = int(rng.choice([32, 64, 96, 160]))
        B = int(rng.choice([1, 2, 31, 33, 64, 65, 130, 257]))
        dtype = ["f32", "bf16"][rng.integers(0, 2)]
        if n * r * v * B > 6_000_000 or n * r * r > 300_000:      # keep the oracle to seconds
            continue
        cases.append((family, dtype, B, d, n, r, v))
    return cases


@pytest.mark.parametrize("family,dtype,B,d,n,r,v", draw_cases())
def test_every_operation_on_a_drawn_shape(family, dtype, B, d, n, r, v):
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=n * 1000 + r * 7 + v, h_scale=1.0)
    head = make_head(inp)
    layers = inp.layers if inp.layers is not None and inp.layers.size else None
    logphi, logw, loglayers = oc._params(family, inp.h, inp.W, inp.Wsum, layers)
    tg = torch.from_numpy(inp.targets).cuda()
    # likelihoods and prefix marginals
    want = oc.prefix_marginals_from(family, logphi, logw, loglayers, inp.targets)
    tol_check(head.prefix_marginals(tg).cpu().numpy(), want, dtype, "prefix marginals")
    tol_check(head.loglik(tg).cpu().numpy(), want[:, -1], dtype, "loglik")
    # drafts, their scores, the table
    S = 2
    nl = oc.n_latents(family, n)
    u = philox.uniforms(B, S, n + nl, seed=9)
    od, ol, margin = oc.sample_from(family, logphi, logw, loglayers, u, with_margin=True)
    table = torch.empty(B, n, r, v, dtype=torch.float32, device="cuda")
    gd, gl, gp = head.sample(S, seed=9, want_prefix=True, logphi=table)
    compare_drafts(gd, gl, od, ol, margin)
    tol_check(table.cpu().numpy(), logphi, dtype, "table")
    scores = oc.prefix_marginals_from(family, logphi, logw, loglayers, gd[:, 0].cpu().numpy())
    tol_check(gp[:, 0].cpu().numpy(), scores, dtype, "draft scores")
    # the same drafts without the table (batches above 64 positions then draw through buckets), and
    # windows scored two sets at a time from W, or from the table
    gd2, gl2, _ = head.sample(S, seed=9)
    compare_drafts(gd2, gl2, od, ol, margin)
    both = head.window_scores(tg.view(B, 1, n), gd2, prefix=True).cpu().numpy()
    tol_check(both[:, 0], want, dtype, "prefix marginals (two window sets)")
    tol_check(both[:, 1], oc.prefix_marginals_from(family, logphi, logw, loglayers, gd2[:, 0].cpu().numpy()), dtype,
              "draft scores (two window sets)")
    tol_check(head.table_scores(table, tg).cpu().numpy(), want[:, -1], dtype, "loglik from the table")
    # univariate marginals, through the table of input units and mixed in registers: a few tokens of
    # every position of two rows against the definition (that one variable observed, the others summed
    # out), and every distribution sums to one
    rows = np.unique([0, B - 1])
    ids = np.unique(np.concatenate([[0, v - 1], np.random.default_rng(3).integers(0, v, size=6)]))
    wins = np.full((len(rows), n, len(ids), n), -1, dtype=np.int64)
    for i in range(n):
        wins[:, i, :, i] = ids[None, :]
    for keep in (True, False):
        M = head.univariate_marginals(keep_table=keep).cpu().numpy()
        for k, b in enumerate(rows):
            x = wins[k].reshape(-1, n)
            rep = lambda t: None if t is None else np.repeat(t[b:b + 1], len(x), axis=0)
            lay_b = loglayers[b] if (loglayers is not None and loglayers.ndim == 4) else loglayers
            want_u = oc.joint(family, oc.evidence(rep(logphi), x), rep(logw), lay_b).reshape(n, len(ids))
            tol_check(M[b][:, ids], want_u, dtype, f"univariate marginals (table kept: {keep})")
        assert np.abs(np.log(np.exp(M.astype(np.float64)).sum(axis=-1))).max() < 2e-4
    # verification on oracle-built inputs
    drafts = od[:, 0].astype(np.int32)
    P = oc.prefix_marginals_from(family, logphi, logw, loglayers, drafts)
    p = synthetic_verifier(inp, logphi, logw, loglayers, drafts, seed=4)
    uv = philox.verify_uniforms(B, n + 1, 10, 1)
    w_acc, w_tok, mg = sp.speculative_verify(family, logphi, logw, loglayers, drafts, p, uv)
    acc, tok = head.verify(torch.from_numpy(drafts).cuda(), torch.from_numpy(p.astype(np.float32)).cuda(),
                           prefix_logq=torch.from_numpy(P.astype(np.float32)).cuda(),
                           logphi=torch.from_numpy(logphi.astype(np.float32)).cuda(), seed=10, offset=1)
    safe = mg >= 2e-5
    assert np.array_equal(acc.cpu().numpy()[safe], w_acc[safe]) and np.array_equal(tok.cpu().numpy()[safe], w_tok[safe])
    # training step
    coef = bw.loss_coefficients(0.9, np.random.default_rng(2).random((B, n)) > 0.1).astype(np.float32)
    out = head.loss_backward(tg, torch.from_numpy(coef).cuda())
    ref = bw.loss_and_gradients(family, inp.h, inp.W, inp.Wsum, layers, inp.targets, coef)
    for name in ("dh", "dW", "dWsum", "dlayers"):
        if ref[name] is None:
            continue
        got = out[name].cpu().numpy().astype(np.float64)
        scale = max(np.abs(ref[name]).max(), 1e-30)
        # fp32 paths: 1e-4 of the largest entry.  The softmax-backward differences G - omega sum(G)
        # behind dWsum and dlayers lose about three digits to cancellation, after a reverse chain of
        # `steps` fp32 products (7 n for the tree's program, n for the HMM): 2^-24 * 1e3 * sqrt(steps),
        # i.e. 6e-5 sqrt(steps), at least 5e-4 (1.3e-3 for the 446 steps of a tree over 64 tokens)
        steps = {"btree": 7 * n, "hmm": n}.get(family, 1)
        lim_sum = max(5e-4, 6e-5 * np.sqrt(steps))
        lim = (lim_sum if name in ("dWsum", "dlayers") else 1e-4) if (dtype == "f32" or name == "dlayers") else 2e-2
        # floor: with a one-token vocabulary every gradient is exactly zero and only the rounding of
        # the fp32 sums is left, one unit in the last place of their largest summands: the coefficients
        # of all windows times the largest |h| (1.9e-7 seen for a tree over 16 tokens at B = 1)
        floor = max(1e-7, 2.0 ** -23 * float(coef.sum()) * float(np.abs(inp.h.astype(np.float64)).max()))
        assert np.abs(got - ref[name]).max() <= lim * scale + floor, (name, np.abs(got - ref[name]).max() / scale)
