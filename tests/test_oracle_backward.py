"""Pins for the oracle of the training step (Sec. 4.1 loss, gradients), no GPU.

The differentiated forward pass is checked against the NumPy oracle, its
gradients against central finite differences of a loss that only the NumPy
oracle evaluates, against the textbook cross-entropy gradient in the fully
factorised case, and the loss coefficients against a table worked out by hand."""
import numpy as np
import pytest

from oracle import backward as bw
from oracle import mtpc_oracle as oc

from test_oracle_circuits import tiny

FAMS = ("ff", "cp", "hmm", "btree")


def numpy_loss(family, h, W, Wsum, layers, targets, coef):
    P = oc.prefix_marginals(family, h, W, Wsum, layers, targets)
    prev = np.concatenate([np.zeros((P.shape[0], 1)), P[:, :-1]], axis=1)
    return float((coef * (prev - P)).sum())


def setup(family, n=4, r=3, v=4, d=5, B=3, seed=0):
    h, W, Wsum, layers = tiny(family, n, r, v, d=d, B=B, seed=seed)
    rng = np.random.default_rng(seed + 100)
    targets = rng.integers(0, v, size=(B, n))
    coef = rng.random((B, n)) * (rng.random((B, n)) > 0.2)
    return h, W, Wsum, layers, targets, coef


@pytest.mark.parametrize("family", FAMS)
def test_differentiated_forward_equals_numpy_oracle(family):
    h, W, Wsum, layers, targets, coef = setup(family, n=8, r=4, v=6)
    res = bw.loss_and_gradients(family, h, W, Wsum, layers, targets, coef)
    want = oc.prefix_marginals(family, h, W, Wsum, layers, targets)
    np.testing.assert_allclose(res["P"], want, rtol=0, atol=1e-11)
    assert abs(res["loss"].sum() - numpy_loss(family, h, W, Wsum, layers, targets, coef)) < 1e-10


@pytest.mark.parametrize("family", FAMS)
def test_gradients_equal_finite_differences_of_the_numpy_loss(family):
    h, W, Wsum, layers, targets, coef = setup(family, seed=3)
    res = bw.loss_and_gradients(family, h, W, Wsum, layers, targets, coef)
    rng = np.random.default_rng(7)
    eps = 1e-6
    params = {"dh": h, "dW": W, "dWsum": Wsum, "dlayers": layers}
    for name, arr in params.items():
        if arr is None:
            assert res[name] is None
            continue
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            up = numpy_loss(family, h, W, Wsum, layers, targets, coef)
            arr[idx] = old - eps
            dn = numpy_loss(family, h, W, Wsum, layers, targets, coef)
            arr[idx] = old
            fd = (up - dn) / (2 * eps)
            assert abs(fd - res[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, res[name][idx])


@pytest.mark.parametrize("family", FAMS)
def test_summed_out_targets_follow_the_numpy_oracle(family):
    h, W, Wsum, layers, targets, coef = setup(family, seed=4)
    targets[0, 1] = targets[2, 3] = targets[1, 0] = -1
    res = bw.loss_and_gradients(family, h, W, Wsum, layers, targets, coef)
    np.testing.assert_allclose(res["P"], oc.prefix_marginals(family, h, W, Wsum, layers, targets), atol=1e-11)
    eps, rng = 1e-6, np.random.default_rng(2)
    for _ in range(10):
        idx = tuple(rng.integers(0, s) for s in W.shape)
        old = W[idx]
        W[idx] = old + eps
        up = numpy_loss(family, h, W, Wsum, layers, targets, coef)
        W[idx] = old - eps
        dn = numpy_loss(family, h, W, Wsum, layers, targets, coef)
        W[idx] = old
        assert abs((up - dn) / (2 * eps) - res["dW"][idx]) <= 1e-6
    # no gradient reaches the unembedding rows of a summed-out position of a one-position batch
    one = bw.loss_and_gradients(family, h[:1], W, Wsum, layers, targets[:1], coef[:1])
    assert np.abs(one["dW"][1]).max() == 0.0


def test_layers_computed_from_the_hidden_state_match_finite_differences():
    """Contextual HMM (Sec. 3.3, App. HMM setup): transition logits R h + bias."""
    h, W, Wsum, bias, targets, coef = setup("hmm", seed=6)
    n, r, d = W.shape[0], W.shape[1], h.shape[1]
    R = np.random.default_rng(8).standard_normal((n - 1, r, r, d)) * 0.7
    res = bw.loss_and_gradients("hmm", h, W, Wsum, bias, targets, coef, R=R)

    def f():
        lay = oc.contextual_layer_logits(h, R, bias)
        return numpy_loss("hmm", h, W, Wsum, lay, targets, coef)
    np.testing.assert_allclose(res["P"], oc.prefix_marginals("hmm", h, W, Wsum, oc.contextual_layer_logits(h, R, bias),
                                                             targets), atol=1e-11)
    eps, rng = 1e-6, np.random.default_rng(3)
    for name, arr in (("dR", R), ("dlayers", bias), ("dh", h)):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            up = f()
            arr[idx] = old - eps
            dn = f()
            arr[idx] = old
            fd = (up - dn) / (2 * eps)
            assert abs(fd - res[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx)


def test_fully_factorised_gradient_is_softmax_minus_one_hot():
    """-log softmax(l)[x] has gradient softmax(l) - onehot(x) in l = W h (textbook)."""
    h, W, _, _, targets, coef = setup("ff", n=3, r=1, v=5, d=4, B=6, seed=9)
    res = bw.loss_and_gradients("ff", h, W, None, None, targets, coef)
    logits = np.einsum("nrvd,bd->bnrv", W, h)[:, :, 0]                     # [B,n,v]
    sm = np.exp(logits - logits.max(-1, keepdims=True))
    sm /= sm.sum(-1, keepdims=True)
    onehot = np.eye(W.shape[2])[targets]
    dl = coef[:, :, None] * (sm - onehot)                                   # [B,n,v]
    np.testing.assert_allclose(res["dW"][:, 0], np.einsum("bnv,bd->nvd", dl, h), atol=1e-12)
    np.testing.assert_allclose(res["dh"], np.einsum("bnv,nvd->bd", dl, W[:, 0]), atol=1e-12)
    # every row of the logit gradient sums to zero: h-gradient is orthogonal to a shared shift of W
    assert np.abs(dl.sum(-1)).max() < 1e-12


@pytest.mark.parametrize("family", FAMS)
def test_unit_coefficients_telescope_to_the_log_likelihood(family):
    h, W, Wsum, layers, targets, _ = setup(family, seed=5)
    res = bw.loss_and_gradients(family, h, W, Wsum, layers, targets, np.ones(targets.shape))
    want = -oc.loglik(family, h, W, Wsum, layers, targets)
    np.testing.assert_allclose(res["loss"], want, atol=1e-11)


def test_cp_with_one_component_has_the_fully_factorised_gradient():
    h, W, Wsum, _, targets, coef = setup("cp", r=1, seed=2)
    a = bw.loss_and_gradients("cp", h, W, Wsum, None, targets, coef)
    b = bw.loss_and_gradients("ff", h, W, None, None, targets, coef)
    np.testing.assert_allclose(a["dW"], b["dW"], atol=1e-12)
    np.testing.assert_allclose(a["dh"], b["dh"], atol=1e-12)
    assert np.abs(a["dWsum"]).max() < 1e-12


def test_loss_coefficients_by_hand():
    """Two sequences; gamma = 0.8; slot 0 valid everywhere, slot 1 not at each sequence's end."""
    valid = np.array([[1, 1], [1, 1], [1, 0],      # sequence 0: V = (3, 2)
                      [1, 1], [1, 0]], dtype=bool)  # sequence 1: V = (2, 1)
    seq = np.array([0, 0, 0, 1, 1])
    c = bw.loss_coefficients(0.8, valid, seq)
    want = np.array([[1 / 6, 0.8 / 4], [1 / 6, 0.8 / 4], [1 / 6, 0.0],
                     [1 / 4, 0.8 / 2], [1 / 4, 0.0]])
    np.testing.assert_allclose(c, want, atol=1e-15)
    # one sequence, everything valid: gamma^j / B
    np.testing.assert_allclose(bw.loss_coefficients(0.9, np.ones((4, 3), bool)),
                               np.tile(0.9 ** np.arange(3) / 4, (4, 1)), atol=1e-15)
