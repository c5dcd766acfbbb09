"""GPU parity at the full sizes of the named workloads, in the launch
configuration bench.py times.  The oracle evaluates a fixed sample of positions
(first tile, last tile, random rows); positions are independent, so every sampled
output is computed by the oracle exactly as in the small tests."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi
from oracle import mtpc_oracle as oc
from oracle import philox

from oracle import backward as bw
from oracle import speculative as sp

from gpu_util import BOUNDARY, compare_drafts, make_head, synthetic_verifier, tol_check

pytestmark = pytest.mark.gpu


def sample_rows(B, k=40, seed=0):
    rng = np.random.default_rng(seed)
    rows = set(range(0, 6)) | set(range(B - 6, B)) | set(rng.integers(0, B, size=k).tolist())
    rows |= {255, 256, 257} & set(range(B))
    return np.array(sorted(rows))


def check_rows(inp, head, rows, S=0, seed=0):
    tg = torch.from_numpy(inp.targets).cuda()
    gP = head.prefix_marginals(tg).cpu().numpy()
    gL = head.loglik(tg).cpu().numpy()
    lay = inp.layers
    if inp.R is not None:            # layers computed from h: R h + bias
        lay = oc.contextual_layer_logits(inp.h[rows], inp.R, inp.layers)
    logphi, logw, loglayers = oc._params(inp.family, inp.h[rows], inp.W,
                                         inp.Wsum, lay)
    want = oc.prefix_marginals_from(inp.family, logphi, logw, loglayers, inp.targets[rows])
    err = tol_check(gP[rows], want, inp.dtype, "prefix marginals")
    tol_check(gL[rows], want[:, -1], inp.dtype, "loglik")
    assert np.array_equal(gL, gP[:, -1])
    assert np.all(np.isfinite(gL)) and np.all(np.diff(gP, axis=1) <= 1e-4)
    print(f"{inp.family} B={inp.B} r={inp.r}: {len(rows)} rows checked, max abs err {err:.2e}")
    if S:
        gd, gl, gp = head.sample(S, seed=seed, want_prefix=True)
        nl = oc.n_latents(inp.family, inp.n)
        u_all = philox.uniforms(inp.B, S, inp.n + nl, seed)
        od, ol, margin = oc.sample_from(inp.family, logphi, logw, loglayers, u_all[rows], with_margin=True)
        near, bad = compare_drafts(gd[rows], gl[rows] if gl is not None else None, od, ol, margin)
        print(f"  drafts: {near} of {margin.size} within {BOUNDARY} of a CDF step, {bad} of those differ")
        gdn = gd.cpu().numpy()
        for s in range(S):
            ps = oc.prefix_marginals_from(inp.family, logphi, logw, loglayers, gdn[rows, s])
            tol_check(gp[rows, s].cpu().numpy(), ps, inp.dtype, "draft scores")
        # the step bench.py times: drafts alone, then targets and drafts scored in one fused pass
        gd2, _, _ = head.sample(S, seed=seed)
        assert torch.equal(gd2, gd)
        both = head.window_scores(tg.view(inp.B, 1, inp.n), gd2, prefix=True).cpu().numpy()
        tol_check(both[rows, 0], want, inp.dtype, "prefix marginals of the targets (fused with the drafts)")
        for s in range(S):
            ps = oc.prefix_marginals_from(inp.family, logphi, logw, loglayers, gdn[rows, s])
            tol_check(both[rows, 1 + s], ps, inp.dtype, "draft scores (fused with the targets)")


def test_config2_ff_and_cp16_full_size():
    for r in (1, 16):
        inp = mi.config2(r=r)
        head = make_head(inp)
        check_rows(inp, head, sample_rows(inp.B), S=1 if r == 16 else 0)
        del head
        torch.cuda.empty_cache()


def test_config3_hmm_full_size():
    inp = mi.config3()
    head = make_head(inp)
    check_rows(inp, head, sample_rows(inp.B, k=24), S=1, seed=2)
    univariate_rows(inp, head, np.array([0, 300, inp.B - 1]))


def test_config3_contextual_hmm_full_size():
    """The paper's own HMM variant: every transition computed from the hidden state."""
    inp = mi.config3_contextual()
    head = make_head(inp)
    check_rows(inp, head, sample_rows(inp.B, k=24), S=1, seed=5)


@pytest.mark.parametrize("family", ["cp", "btree"])
def test_llama_byte_shape_fp32_ragged_vocabulary(family):
    """fp32 MFMA path at scale with v = 268 (masked pad rows), d = 3072."""
    inp = mi.config_llama_byte(family)
    head = make_head(inp)
    check_rows(inp, head, sample_rows(inp.B, k=20), S=1, seed=9)


def univariate_rows(inp, head, rows):
    """Univariate marginals of a few positions against the definition, through the table of input
    units (offsets beyond 2^30 elements at the larger workloads) and mixed in registers; every
    distribution of the batch sums to one."""
    want = oc.univariate_marginals(inp.family, inp.h[rows], inp.W, inp.Wsum, inp.layers)
    for keep in (True, False):
        M = head.univariate_marginals(keep_table=keep)
        err = tol_check(M[rows].cpu().numpy(), want, inp.dtype, f"univariate marginals (table kept: {keep})")
        total = torch.logsumexp(M.double(), dim=-1).abs().max().item()
        assert total < 2e-4, total
        print(f"  univariate (table kept: {keep}): max abs err {err:.2e} on {len(rows)} rows, |log sum| <= {total:.1e}")
        del M


def test_config4_btree_full_size():
    """Loglik + marginals (prefix and univariate) + one draft per position of the 16-leaf tree;
    the targets cover every id of the vocabulary, also the 64 beyond the bytes."""
    inp = mi.config4(targets="uniform")
    assert inp.targets.max() >= 256
    head = make_head(inp)
    check_rows(inp, head, sample_rows(inp.B, k=12), S=1, seed=3)
    univariate_rows(inp, head, np.array([0, inp.B // 2 + 1, inp.B - 1]))


@pytest.mark.parametrize("B", [1, 8, 64])
def test_config5_decode_draft_and_score(B):
    inp = mi.config5(B=B)
    head = make_head(inp)
    check_rows(inp, head, np.arange(B), S=1, seed=0)
    # 16 prefixes of random length per draft, scored from the table the sampling call keeps
    table = torch.empty(B, inp.n, inp.r, inp.v, dtype=torch.float32, device="cuda")
    gd, _, gp = head.sample(1, seed=0, want_prefix=True, logphi=table)
    lens = np.random.default_rng(B).integers(1, inp.n + 1, size=(B, 16))
    x16 = np.repeat(gd.cpu().numpy()[:, :1, :], 16, axis=1)
    x16[np.arange(inp.n)[None, None, :] >= lens[:, :, None]] = -1
    got = head.table_scores(table, torch.from_numpy(x16).cuda()).cpu().numpy()
    logphi, logw, loglayers = oc._params(inp.family, inp.h, inp.W, inp.Wsum, inp.layers)
    P = oc.prefix_marginals_from(inp.family, logphi, logw, loglayers, gd.cpu().numpy()[:, 0])
    tol_check(got, np.take_along_axis(P, lens - 1, axis=1), inp.dtype, "16 prefixes per draft")


def test_config5_decode_cycle_with_verification():
    """Draft, score, keep the input-unit table, verify (Alg. 2) at the decode shape."""
    inp = mi.config5(B=64)
    B, n, r, v = inp.B, inp.n, inp.r, inp.v
    head = make_head(inp)
    logphi, logw, loglayers = oc._params(inp.family, inp.h, inp.W, inp.Wsum, inp.layers)
    table = torch.empty(B, n, r, v, dtype=torch.float32, device="cuda")
    gd, _, gp = head.sample(1, seed=4, want_prefix=True, logphi=table)
    tol_check(table.cpu().numpy(), logphi, inp.dtype, "log phi table")
    od, _ = oc.sample_from(inp.family, logphi, logw, loglayers, philox.uniforms(B, 1, n + 1, 4, 0))
    drafts = od[:, 0].astype(np.int32)
    p = synthetic_verifier(inp, logphi, logw, loglayers, drafts, seed=8)
    u = philox.verify_uniforms(B, n + 1, 21, 1)
    want_acc, want_tok, margin = sp.speculative_verify(inp.family, logphi, logw, loglayers, drafts, p, u)
    gdn = gd[:, 0].contiguous()
    acc, tok = head.verify(gdn, torch.from_numpy(p.astype(np.float32)).cuda(), prefix_logq=gp[:, 0].contiguous(),
                           logphi=table, seed=21, offset=1)
    safe = np.all(gdn.cpu().numpy() == drafts, axis=1) & (margin >= 4e-3)
    assert np.array_equal(acc.cpu().numpy()[safe], want_acc[safe])
    assert np.array_equal(tok.cpu().numpy()[safe], want_tok[safe])
    print(f"accepted histogram {np.bincount(want_acc, minlength=n + 1)}; {int((~safe).sum())} of {B} rows near a boundary")
    assert safe.sum() >= B // 2 and len(np.unique(want_acc)) >= 4
    # the kernel alone at this shape: draft, scores and table from the oracle, so only rows whose
    # decisions lie within fp32 rounding (2e-5) of their boundary are left out
    P = oc.prefix_marginals_from(inp.family, logphi, logw, loglayers, drafts)
    acc3, tok3 = head.verify(torch.from_numpy(drafts).cuda(), torch.from_numpy(p.astype(np.float32)).cuda(),
                             prefix_logq=torch.from_numpy(P.astype(np.float32)).cuda(),
                             logphi=torch.from_numpy(logphi.astype(np.float32)).cuda(), seed=21, offset=1)
    exact = margin >= 2e-5
    assert np.array_equal(acc3.cpu().numpy()[exact], want_acc[exact])
    assert np.array_equal(tok3.cpu().numpy()[exact], want_tok[exact])
    print(f"oracle-built inputs: {int(exact.sum())} of {B} rows compared bit-exact")
    assert exact.sum() >= B - 4


def test_config2_training_step_full_size():
    """Loss and gradients of configs[1] (CP r=16, B=8192) in the launch configuration the
    bench times.  dh and the loss are per-position quantities: sampled rows against the
    oracle.  dW sums over all positions: (1) exact comparison of every entry in a second
    run whose coefficients are zero outside a few dozen positions (the oracle differentiates
    those alone), (2) on the dense run the identities sum_a dW[i,j,a,:] = 0 (softmax rows of
    the logit gradient sum to zero) and <dh,h> = <dW,W> + <dWsum,Wsum> (both sides are the
    logit gradient contracted with the logits)."""
    inp = mi.config2(r=16)
    B, n = inp.B, inp.n
    head = make_head(inp)
    rng = np.random.default_rng(12)
    valid = rng.random((B, n)) > 0.1
    coef = bw.loss_coefficients(0.8, valid, sequence=np.arange(B) // 1024).astype(np.float32)
    tg = torch.from_numpy(inp.targets).cuda()
    out = head.loss_backward(tg, torch.from_numpy(coef).cuda())
    rows = sample_rows(B, k=12)
    want = bw.loss_and_gradients("cp", inp.h[rows], inp.W, inp.Wsum, None, inp.targets[rows], coef[rows])
    dh = out["dh"].cpu().numpy()[rows].astype(np.float64)
    fro = np.linalg.norm(dh - want["dh"]) / np.linalg.norm(want["dh"])
    assert fro <= 3e-3 and np.abs(dh - want["dh"]).max() <= 2e-2 * np.abs(want["dh"]).max(), fro
    loss = out["loss"].cpu().numpy()[rows]
    assert np.all(np.abs(loss - want["loss"]) <= 2e-3 * np.maximum(np.abs(want["loss"]), 1e-6))
    dW, dWs = out["dW"].double(), out["dWsum"].double()
    scale = float(dW.abs().max())
    # 320 bf16-rounded terms per sum: random error about 2^-9 * sqrt(320) of a typical entry
    assert float(dW.sum(dim=2).abs().max()) <= 0.1 * scale
    Wd = torch.from_numpy(inp.W).cuda().double()
    lhs = float((out["dh"].double() * torch.from_numpy(inp.h).cuda().double()).sum())
    rhs = float((dW * Wd).sum()) + float((dWs * torch.from_numpy(inp.Wsum).cuda().double()).sum())
    assert abs(lhs - rhs) <= 3e-3 * max(abs(lhs), float((dW * Wd).abs().sum()) * 1e-3), (lhs, rhs)
    print(f"dense run: dh rows rel. Frobenius error {fro:.1e}; <dh,h> = {lhs:.6e}, <dW,W>+<dWsum,Wsum> = {rhs:.6e}")
    del dW, dWs, Wd

    few = np.unique(np.concatenate([sample_rows(B, k=16, seed=3), [4095, 4096, B - 1]]))
    sparse = np.zeros_like(coef)
    sparse[few] = coef[few] * 100.0
    out2 = head.loss_backward(tg, torch.from_numpy(sparse).cuda(), out=out)
    want2 = bw.loss_and_gradients("cp", inp.h[few], inp.W, inp.Wsum, None, inp.targets[few], sparse[few])
    for name in ("dW", "dWsum"):
        got = out2[name].cpu().numpy().astype(np.float64)
        err = np.abs(got - want2[name])
        fro2 = np.linalg.norm(got - want2[name]) / np.linalg.norm(want2[name])
        assert fro2 <= 3e-3 and err.max() <= 2e-2 * np.abs(want2[name]).max(), (name, fro2)
        print(f"sparse run ({len(few)} positions): {name} rel. Frobenius error {fro2:.1e}")
    others = np.setdiff1d(np.arange(B), few)
    assert float(out2["dh"][torch.from_numpy(others).cuda()].abs().max()) == 0.0


def test_config4_training_step_full_size():
    """Training step of configs[3] (binary tree, r = 64, n = 16, B = 4096) in the launch
    configuration the bench times.  One oracle call differentiates a dozen positions: the dense
    run's loss and dh are compared on those positions; a second run whose coefficients vanish
    elsewhere (and are 100 times larger there: the gradients are linear in them) gives dW, dWsum
    and the gradient of the 14 shared layers entry by entry.  The dense run also has to satisfy
    sum_a dW[i,j,a,:] = 0 and <dh,h> = <dW,W> + <dWsum,Wsum> (static layers do not depend on h)."""
    inp = mi.config4()
    B, n = inp.B, inp.n
    head = make_head(inp)
    rng = np.random.default_rng(14)
    valid = rng.random((B, n)) > 0.1
    coef = bw.loss_coefficients(0.8, valid, sequence=np.arange(B) // 1024).astype(np.float32)
    tg = torch.from_numpy(inp.targets).cuda()
    out = head.loss_backward(tg, torch.from_numpy(coef).cuda())
    few = np.unique(np.concatenate([sample_rows(B, k=8, seed=4), [2047, 2048, B - 1]]))
    want = bw.loss_and_gradients("btree", inp.h[few], inp.W, inp.Wsum, inp.layers, inp.targets[few], coef[few])
    dh = out["dh"].cpu().numpy()[few].astype(np.float64)
    fro = np.linalg.norm(dh - want["dh"]) / np.linalg.norm(want["dh"])
    assert fro <= 3e-3 and np.abs(dh - want["dh"]).max() <= 2e-2 * np.abs(want["dh"]).max(), fro
    loss = out["loss"].cpu().numpy()[few]
    assert np.all(np.abs(loss - want["loss"]) <= 2e-3 * np.maximum(np.abs(want["loss"]), 1e-6))
    dW = out["dW"]
    scale = float(dW.abs().max())
    assert float(dW.sum(dim=2, dtype=torch.float64).abs().max()) <= 0.1 * scale
    Wg, hg = torch.from_numpy(inp.W).cuda(), torch.from_numpy(inp.h).cuda()
    lhs = float((out["dh"].double() * hg.double()).sum())
    dWW = [float((dW[i].double() * Wg[i].double()).sum()) for i in range(n)]
    absW = sum(float((dW[i].double() * Wg[i].double()).abs().sum()) for i in range(n))
    rhs = sum(dWW) + float((out["dWsum"].double() * torch.from_numpy(inp.Wsum).cuda().double()).sum())
    assert abs(lhs - rhs) <= 3e-3 * max(abs(lhs), absW * 1e-3), (lhs, rhs)
    print(f"dense run: dh rows rel. Frobenius error {fro:.1e}; <dh,h> = {lhs:.6e}, <dW,W>+<dWsum,Wsum> = {rhs:.6e}")
    del Wg, hg, dW

    sparse = np.zeros_like(coef)
    sparse[few] = coef[few] * 100.0
    out2 = head.loss_backward(tg, torch.from_numpy(sparse).cuda(), out=out)
    got = out2["dlayers"].cpu().numpy().astype(np.float64)
    ref = 100.0 * want["dlayers"]
    f2 = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert f2 <= 3e-3 and np.abs(got - ref).max() <= 2e-2 * np.abs(ref).max(), f2
    print(f"sparse run ({len(few)} positions): dlayers rel. Frobenius error {f2:.1e}")
    # The gradient of a sum-unit logit is c * (posterior_z - omega_z) summed over the prefixes.  Behind
    # fourteen random 64 x 64 layers the root's latent hardly depends on the tokens: the posterior is
    # omega to four or five digits, and the difference of two fp32 numbers of size c * omega keeps
    # an absolute error of a few units of THEIR last place, not of its own.  So the bound is the
    # relative one plus 8 fp32 units (2^-23) of the terms that cancel, sum_b |c_b| omega_bz |h_bd|.
    hs = inp.h[few].astype(np.float64)
    z = hs @ inp.Wsum.astype(np.float64).T
    omega = np.exp(z - z.max(axis=1, keepdims=True))
    omega /= omega.sum(axis=1, keepdims=True)
    cancel = np.einsum("b,bz,bd->zd", np.abs(sparse[few]).astype(np.float64).sum(axis=1), omega, np.abs(hs))
    got = out2["dWsum"].cpu().numpy().astype(np.float64)
    ref = 100.0 * want["dWsum"]
    err = np.abs(got - ref).max()
    assert err <= 3e-3 * np.abs(ref).max() + 8 * 2.0 ** -23 * cancel.max(), (err, np.abs(ref).max(), cancel.max())
    print(f"sparse run: dWsum max error {err:.1e}, largest entry {np.abs(ref).max():.1e}, "
          f"cancelling terms {cancel.max():.1e}")
    num = den = 0.0
    top = 100.0 * np.abs(want["dW"]).max()
    for i in range(n):                       # token by token: the full array is 8 GB in float64
        got = out2["dW"][i].cpu().numpy().astype(np.float64)
        ref = 100.0 * want["dW"][i]
        assert np.abs(got - ref).max() <= 2e-2 * top, i
        num += float(((got - ref) ** 2).sum())
        den += float((ref ** 2).sum())
    assert np.sqrt(num / den) <= 3e-3, np.sqrt(num / den)
    print(f"sparse run: dW rel. Frobenius error {np.sqrt(num / den):.1e}")
    others = np.setdiff1d(np.arange(B), few)
    assert float(out2["dh"][torch.from_numpy(others).cuda()].abs().max()) == 0.0


def test_config3_contextual_training_step_full_size():
    """The HMM the paper trains (transition logits R h + bias), B = 8192: loss and dh on
    sampled positions against the oracle; dW, dWsum, dR and the bias gradient exactly in a
    run whose coefficients vanish outside a couple of dozen positions."""
    inp = mi.config3_contextual()
    B, n = inp.B, inp.n
    head = make_head(inp)
    coef = bw.loss_coefficients(0.8, np.ones((B, n), bool), sequence=np.arange(B) // 2048).astype(np.float32)
    tg = torch.from_numpy(inp.targets).cuda()
    out = head.loss_backward(tg, torch.from_numpy(coef).cuda())
    rows = sample_rows(B, k=6)
    want = bw.loss_and_gradients("hmm", inp.h[rows], inp.W, inp.Wsum, inp.layers, inp.targets[rows], coef[rows], R=inp.R)
    dh = out["dh"].cpu().numpy()[rows].astype(np.float64)
    fro = np.linalg.norm(dh - want["dh"]) / np.linalg.norm(want["dh"])
    assert fro <= 3e-3, fro
    assert np.all(np.abs(out["loss"].cpu().numpy()[rows] - want["loss"]) <= 2e-3 * np.maximum(np.abs(want["loss"]), 1e-6))
    few = np.unique(np.concatenate([sample_rows(B, k=6, seed=5), [4095, 4096]]))
    sparse = np.zeros_like(coef)
    sparse[few] = coef[few] * 100.0
    out2 = head.loss_backward(tg, torch.from_numpy(sparse).cuda(), out=out)
    want2 = bw.loss_and_gradients("hmm", inp.h[few], inp.W, inp.Wsum, inp.layers, inp.targets[few], sparse[few], R=inp.R)
    msg = [f"dh rows {fro:.1e}"]
    for name in ("dW", "dWsum", "dR", "dlayers"):
        got = out2[name].cpu().numpy().astype(np.float64)
        f2 = np.linalg.norm(got - want2[name]) / np.linalg.norm(want2[name])
        assert f2 <= 3e-3 and np.abs(got - want2[name]).max() <= 2e-2 * np.abs(want2[name]).max(), (name, f2)
        msg.append(f"{name} {f2:.1e}")
    print("relative Frobenius errors:", " ".join(msg))


def test_llama_byte_training_step_fp32_split_k():
    """fp32 training step at the second model shape (d = 3072, v = 268, r = 32, B = 2048): the dh
    contraction has 96 output tiles and runs split over K; vocabulary rows 268..319 of the tile
    are padding.  Sampled rows for dh and the loss, a sparse-coefficient run for dW and dWsum."""
    inp = mi.config_llama_byte("cp")
    B, n = inp.B, inp.n
    head = make_head(inp)
    coef = bw.loss_coefficients(0.9, np.ones((B, n), bool)).astype(np.float32)
    tg = torch.from_numpy(inp.targets).cuda()
    out = head.loss_backward(tg, torch.from_numpy(coef).cuda())
    rows = sample_rows(B, k=6)
    want = bw.loss_and_gradients("cp", inp.h[rows], inp.W, inp.Wsum, None, inp.targets[rows], coef[rows])
    dh = out["dh"].cpu().numpy()[rows].astype(np.float64)
    assert np.abs(dh - want["dh"]).max() <= 2e-5 * np.abs(want["dh"]).max()
    assert np.all(np.abs(out["loss"].cpu().numpy()[rows] - want["loss"]) <= 1e-4 * np.maximum(1.0, np.abs(want["loss"])))
    few = np.unique(np.concatenate([sample_rows(B, k=4, seed=2), [1023, 1024]]))
    sparse = np.zeros_like(coef)
    sparse[few] = coef[few] * 50.0
    out2 = head.loss_backward(tg, torch.from_numpy(sparse).cuda(), out=out)
    want2 = bw.loss_and_gradients("cp", inp.h[few], inp.W, inp.Wsum, None, inp.targets[few], sparse[few])
    for name, tol in (("dW", 2e-5), ("dWsum", 1e-4)):
        # the sum-unit gradient G_z - omega_z sum G is a difference of nearly equal fp32 terms
        got = out2[name].cpu().numpy().astype(np.float64)
        assert np.abs(got - want2[name]).max() <= tol * np.abs(want2[name]).max(), name
    print("fp32 training step: dh rows, loss, dW within 2e-5 and dWsum within 1e-4 of the largest entry")
