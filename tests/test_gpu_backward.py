"""GPU parity of the training step (Sec. 4.1 loss and its gradients) against the
float64 reverse-mode oracle.

Tolerances.  fp32 inputs: the contractions run on the fp32 matrix pipes, so every
gradient entry agrees to 2e-5 of the tensor's largest entry.  bf16 inputs: the
logit gradient is rounded to bf16 (relative 2^-9 per entry, independent signs)
before the two contractions, so a gradient entry carries a random error of about
2^-9 / sqrt(3) times the root-sum-square of its terms: the tensors agree to 3e-3
in the Frobenius norm and every entry to 2e-2 of the largest entry.  The loss is
a combination of prefix log-marginals and keeps their tolerance."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi
from oracle import backward as bw

from gpu_util import make_head

pytestmark = pytest.mark.gpu


def check_grad(name, got, want, dtype):
    got, want = got.cpu().numpy().astype(np.float64), np.asarray(want)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    assert np.all(np.isfinite(got)), name
    err = np.abs(got - want)
    big = np.abs(want).max()
    fro = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    if dtype == "f32":
        assert err.max() <= 2e-5 * big + 1e-9, f"{name}: max err {err.max():.3e} vs scale {big:.3e}"
    else:
        assert fro <= 3e-3, f"{name}: relative Frobenius error {fro:.3e}"
        assert err.max() <= 2e-2 * big, f"{name}: max err {err.max():.3e} vs scale {big:.3e}"
    return fro


def make_case(family, dtype, B, d, n, r, v, seed):
    shared = family.endswith("-shared")                          # one transition matrix for all steps
    ctx = "-ctx" in family                                       # transition logits R h + bias (Sec. 3.3)
    perpos = "-perpos" in family                                 # logits of every position supplied by the caller
    family = family.split("-")[0]
    inp = mi.make_inputs(family, B=B, d=d, n=n, r=r, v=v, dtype=dtype, seed=seed, h_scale=1.0,
                         layer_count=1 if shared else None, contextual=ctx)
    if perpos:
        inp.layers = np.random.default_rng(seed + 7).standard_normal((B,) + inp.layers.shape).astype(np.float32)
    rng = np.random.default_rng(seed + 1)
    targets = inp.targets.copy()
    targets[rng.random(targets.shape) < 0.05] = -1               # a few summed-out variables
    valid = rng.random((B, n)) > 0.15
    coef = bw.loss_coefficients(0.8, valid, sequence=np.arange(B) // max(B // 3, 1))
    return inp, targets.astype(np.int32), coef


CASES = [
    ("ff", "f32", 70, 64, 4, 1, 33, 1),
    ("ff", "bf16", 257, 128, 3, 1, 320, 2),
    ("cp", "f32", 70, 64, 4, 5, 33, 3),
    ("cp", "bf16", 300, 128, 8, 16, 320, 4),
    ("cp", "bf16", 33, 256, 2, 128, 200, 5),
    ("cp", "f32", 1, 32, 1, 3, 7, 6),
    ("hmm", "f32", 70, 64, 4, 5, 33, 7),
    ("hmm", "bf16", 300, 128, 8, 32, 320, 8),
    ("hmm", "bf16", 40, 64, 16, 128, 64, 9),
    ("hmm", "f32", 9, 32, 1, 4, 12, 10),
    ("hmm-shared", "f32", 50, 64, 6, 8, 40, 11),
    ("btree", "f32", 70, 64, 4, 5, 33, 12),
    ("btree", "bf16", 130, 128, 8, 16, 320, 13),
    ("btree", "f32", 21, 32, 2, 6, 20, 14),
    ("btree", "bf16", 37, 64, 16, 128, 40, 15),
    ("btree-shared", "f32", 45, 64, 8, 8, 40, 16),
    ("hmm-ctx", "f32", 70, 64, 4, 5, 33, 17),
    ("hmm-ctx", "bf16", 200, 128, 8, 16, 320, 18),
    ("hmm-ctx", "bf16", 37, 64, 3, 128, 40, 19),
    ("btree-ctx", "f32", 70, 64, 4, 5, 33, 20),
    ("btree-ctx", "bf16", 150, 128, 8, 16, 320, 21),
    ("btree-ctx", "bf16", 20, 64, 16, 128, 24, 22),
    # one R (and bias) shared by all steps / inner nodes
    ("hmm-ctx-shared", "f32", 60, 64, 5, 8, 33, 24),
    ("btree-ctx-shared", "bf16", 90, 64, 8, 16, 100, 25),
    # layer logits given per position by the caller: the gradient has their shape
    ("hmm-perpos", "f32", 50, 64, 4, 6, 33, 26),
    ("btree-perpos", "bf16", 70, 64, 8, 16, 64, 27),
    ("hmm-perpos-shared", "f32", 33, 32, 6, 5, 20, 28),
]


@pytest.mark.parametrize("family,dtype,B,d,n,r,v,seed", CASES)
def test_loss_and_gradients_match_oracle(family, dtype, B, d, n, r, v, seed):
    inp, targets, coef = make_case(family, dtype, B, d, n, r, v, seed)
    family = inp.family
    head = make_head(inp)
    out = head.loss_backward(torch.from_numpy(targets).cuda(), torch.from_numpy(coef.astype(np.float32)).cuda())
    layers = inp.layers if inp.layers is not None and inp.layers.size else None
    want = bw.loss_and_gradients(family, inp.h, inp.W, inp.Wsum, layers, targets, coef.astype(np.float32), R=inp.R)
    loss = out["loss"].cpu().numpy()
    tol = 1e-4 if dtype == "f32" else 2e-3
    assert np.all(np.abs(loss - want["loss"]) <= tol * np.maximum(np.abs(want["loss"]), 1e-2) + (1e-4 if dtype == "f32" else 0))
    msg = [f"{family} {dtype} B={B} n={n} r={r} v={v}:"]
    for name in ("dh", "dW", "dWsum", "dlayers", "dR"):
        if want[name] is None or want[name].size == 0:
            continue
        # gradients of layers shared by all positions never pass through the bf16 logit gradient:
        # fp32 accuracy for both dtypes; with R they do (bias = column sums of rounded values)
        crit = "f32" if (name == "dlayers" and inp.R is None) else dtype
        msg.append(f"{name} {check_grad(name, out[name], want[name], crit):.1e}")
    print(" ".join(msg), "(relative Frobenius error)")
    # a second call with the same buffers gives the same bits (nothing accumulates across calls)
    again = head.loss_backward(torch.from_numpy(targets).cuda(), torch.from_numpy(coef.astype(np.float32)).cuda())
    assert torch.equal(again["dW"], out["dW"]) and torch.equal(again["dh"], out["dh"])
    # the lean plan (logits recomputed instead of probabilities kept) meets the same bar
    lean = head.loss_backward(torch.from_numpy(targets).cuda(), torch.from_numpy(coef.astype(np.float32)).cuda(),
                              recompute=True)
    for name in ("dh", "dW", "dWsum", "dR"):
        if want[name] is not None:
            check_grad(name + " (recompute)", lean[name], want[name], dtype)


def test_strided_hidden_states_and_preallocated_outputs():
    """h rows may be a slice of a wider buffer (ld_h > d); outputs may be reused across calls."""
    from paper_2511_11346_amd import Head
    inp, targets, coef = make_case("cp", "bf16", 90, 64, 4, 8, 100, 23)
    base = make_head(inp)
    wide = torch.zeros(90, 192, dtype=torch.bfloat16, device="cuda")
    wide[:, :64] = base.h
    wide[:, 64:] = 7.0                                   # must never be read
    head = Head("cp", wide[:, :64], base.W, base.Wsum)
    tg, cf = torch.from_numpy(targets).cuda(), torch.from_numpy(coef.astype(np.float32)).cuda()
    ref = base.loss_backward(tg, cf)
    out = head.loss_backward(tg, cf)
    for k in ("loss", "dh", "dW", "dWsum"):
        assert torch.equal(out[k], ref[k]), k
    out["dW"].fill_(3.0)
    again = head.loss_backward(tg, cf, out=out)
    assert torch.equal(again["dW"], ref["dW"])



@pytest.mark.parametrize("family,dtype,B,d,n,r,v", [
    ("hmm-shared", "bf16", 1500, 128, 8, 32, 320),     # one matrix applied by 7 steps, 6 blocks of rows
    ("hmm", "f32", 700, 64, 5, 16, 100),
    ("hmm-ctx", "bf16", 700, 128, 4, 16, 130),         # layers R h + bias: bias gradient = column sums
    ("btree", "bf16", 900, 64, 8, 32, 200),            # a node's layer is applied by several program steps
    ("btree-ctx", "f32", 300, 64, 4, 8, 64),
    ("cp", "bf16", 600, 128, 4, 16, 320),
])
def test_training_step_is_bit_reproducible(family, dtype, B, d, n, r, v):
    """The same inputs twice give the same bits in every output: sums over positions (layer and
    bias gradients, split-K partials) are taken in a fixed order, no float atomics."""
    inp, targets, coef = make_case(family, dtype, B, d, n, r, v, seed=77)
    head = make_head(inp)
    tg = torch.from_numpy(targets).cuda()
    cf = torch.from_numpy(coef.astype(np.float32)).cuda()
    for recompute in (False, True):
        first = {k: (None if t is None else t.clone()) for k, t in head.loss_backward(tg, cf, recompute=recompute).items()}
        for _ in range(3):
            again = head.loss_backward(tg, cf, recompute=recompute)
            for k, t in first.items():
                if t is not None:
                    assert torch.equal(t, again[k]), (k, recompute)
