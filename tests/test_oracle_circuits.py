"""Pins for the CPU oracle's circuit semantics (no GPU).

Each test checks the oracle against something other than itself: brute-force
enumeration of windows and of latent assignments written straight from the
displayed equations, equivalences the paper states, library routines for the
special cases that reduce to them, and the figures the paper prints.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import bruteforce as bf
from oracle import mtpc_oracle as oc

FAMS = ("ff", "cp", "hmm", "btree")


def tiny(family, n, r, v, d=5, B=2, seed=0, homogeneous=False):
    rng = np.random.default_rng(seed)
    if family == "ff":
        r = 1
    h = rng.standard_normal((B, d))
    W = rng.standard_normal((n, r, v, d))
    Wsum = None if family == "ff" else rng.standard_normal((r, d))
    layers = None
    if family == "hmm":
        layers = rng.standard_normal((1 if homogeneous else n - 1, r, r)) * 1.5
    if family == "btree":
        layers = rng.standard_normal((n - 2, r, r)) * 1.5
    return h, W, Wsum, layers


def tables(family, h, W, Wsum, layers, b):
    """Explicit linear-domain probability tables of position b, computed with
    torch (a second softmax implementation) for the brute-force evaluators."""
    ht = torch.tensor(h[b], dtype=torch.float64)
    phi = torch.softmax(torch.einsum("nrvd,d->nrv", torch.tensor(W, dtype=torch.float64), ht), dim=-1).numpy()
    omega = None
    if Wsum is not None:
        omega = torch.softmax(torch.tensor(Wsum, dtype=torch.float64) @ ht, dim=-1).numpy()
    lay = None
    if layers is not None:
        lay = torch.softmax(torch.tensor(layers, dtype=torch.float64), dim=-1).numpy()
        n = W.shape[0]
        need = n - 1 if family == "hmm" else n - 2
        if lay.shape[0] == 1 and need > 1:
            lay = np.repeat(lay, need, axis=0)
    return phi, omega, lay


# ---------------------------------------------------------------- normalisation
@pytest.mark.parametrize("family,n,r,v", [
    ("ff", 4, 1, 3), ("cp", 4, 3, 3), ("cp", 8, 2, 2), ("hmm", 4, 3, 3), ("hmm", 8, 2, 2),
    ("hmm", 1, 3, 5), ("btree", 4, 3, 3), ("btree", 8, 2, 2), ("btree", 2, 3, 4),
])
def test_joint_sums_to_one_over_all_windows(family, n, r, v):
    """Circuits are normalised by construction (Sec. 3.1, App. B.1): Z = 1."""
    h, W, Wsum, layers = tiny(family, n, r, v, B=2, seed=n * 100 + r * 10 + v)
    wins = np.array(list(itertools.product(range(v), repeat=n)), dtype=np.int64)
    for b in range(2):
        hb = np.repeat(h[b:b + 1], len(wins), axis=0)
        ll = oc.loglik(family, hb, W, Wsum, layers, wins)
        assert abs(np.exp(ll).sum() - 1.0) < 1e-12


# ------------------------------------------------- recursions vs the equations
@pytest.mark.parametrize("family,n,r,v", [
    ("ff", 5, 1, 4), ("cp", 5, 3, 4), ("hmm", 4, 3, 3), ("hmm", 5, 2, 3),
    ("btree", 4, 3, 3), ("btree", 8, 2, 3), ("btree", 2, 3, 3),
])
def test_joint_equals_latent_enumeration(family, n, r, v):
    h, W, Wsum, layers = tiny(family, n, r, v, B=3, seed=7 + n + r)
    rng = np.random.default_rng(1)
    x = rng.integers(0, v, size=(3, n))
    ll = oc.loglik(family, h, W, Wsum, layers, x)
    for b in range(3):
        phi, omega, lay = tables(family, h, W, Wsum, layers, b)
        p = bf.prob(family, phi, omega, lay, tuple(x[b]))
        assert abs(ll[b] - np.log(p)) < 1e-12 * max(1.0, abs(ll[b]))


def test_homogeneous_hmm_shares_one_transition():
    h, W, Wsum, layers = tiny("hmm", 4, 3, 3, seed=3, homogeneous=True)
    assert layers.shape[0] == 1
    x = np.array([[0, 2, 1, 1], [2, 2, 0, 1]])
    ll = oc.loglik("hmm", h, W, Wsum, layers, x)
    rep = np.repeat(layers, 3, axis=0)
    assert np.allclose(ll, oc.loglik("hmm", h, W, Wsum, rep, x), rtol=0, atol=1e-14)
    for b in range(2):
        phi, omega, lay = tables("hmm", h, W, Wsum, layers, b)
        assert abs(ll[b] - np.log(bf.hmm_prob(phi, omega, lay, tuple(x[b])))) < 1e-12


def test_contextual_layers_use_each_positions_own_matrix():
    h, W, Wsum, _ = tiny("hmm", 3, 2, 3, B=3, seed=11)
    rng = np.random.default_rng(5)
    ctx = rng.standard_normal((3, 2, 2, 2))
    x = rng.integers(0, 3, size=(3, 3))
    ll = oc.loglik("hmm", h, W, Wsum, ctx, x)
    for b in range(3):
        one = oc.loglik("hmm", h[b:b + 1], W, Wsum, ctx[b], x[b:b + 1])
        assert abs(ll[b] - one[0]) < 1e-13


# ----------------------------------------------------- equivalences (paper)
def test_cp_rank_one_is_ff():
    """CP with r = 1 is the fully factorised model (Sec. 4, draft models)."""
    h, W, _, _ = tiny("ff", 6, 1, 7, B=4, seed=2)
    Wsum = np.random.default_rng(0).standard_normal((1, h.shape[1]))
    x = np.random.default_rng(1).integers(0, 7, size=(4, 6))
    a = oc.loglik("ff", h, W, None, None, x)
    b = oc.loglik("cp", h, W, Wsum, None, x)
    assert np.allclose(a, b, rtol=0, atol=1e-13)


@pytest.mark.parametrize("off", [-np.inf, -60.0])
def test_hmm_identity_transitions_is_cp(off):
    """Identity transition matrices make the HMM equal to CP (App. HMM setup)."""
    n, r, v = 5, 4, 6
    h, W, Wsum, _ = tiny("cp", n, r, v, B=4, seed=4)
    eye = np.full((n - 1, r, r), off)
    eye[:, np.arange(r), np.arange(r)] = 0.0
    x = np.random.default_rng(2).integers(0, v, size=(4, n))
    a = oc.loglik("cp", h, W, Wsum, None, x)
    b = oc.loglik("hmm", h, W, Wsum, eye, x)
    assert np.all(np.isfinite(b))
    assert np.allclose(a, b, rtol=0, atol=1e-12)


def test_btree_identity_layers_and_n2_are_cp():
    n, r, v = 8, 3, 4
    h, W, Wsum, _ = tiny("cp", n, r, v, B=3, seed=6)
    eye = np.full((n - 2, r, r), -np.inf)
    eye[:, np.arange(r), np.arange(r)] = 0.0
    x = np.random.default_rng(3).integers(0, v, size=(3, n))
    assert np.allclose(oc.loglik("cp", h, W, Wsum, None, x),
                       oc.loglik("btree", h, W, Wsum, eye, x), rtol=0, atol=1e-12)
    h2, W2, Wsum2, _ = tiny("cp", 2, r, v, B=3, seed=8)
    x2 = x[:, :2]
    assert np.allclose(oc.loglik("cp", h2, W2, Wsum2, None, x2),
                       oc.loglik("btree", h2, W2, Wsum2, np.zeros((0, r, r)), x2), rtol=0, atol=1e-13)


def test_hmm_single_step_is_mixture_of_categoricals():
    h, W, Wsum, _ = tiny("cp", 1, 4, 6, B=3, seed=9)
    x = np.array([[1], [5], [0]])
    a = oc.loglik("hmm", h, W, Wsum, np.zeros((0, 4, 4)), x)
    for b in range(3):
        phi, omega, _ = tables("cp", h, W, Wsum, None, b)
        assert abs(a[b] - np.log(np.dot(omega, phi[0][:, x[b, 0]]))) < 1e-13


def test_ff_is_summed_cross_entropy():
    """FF log-likelihood = minus the summed per-position cross-entropy of the
    logits h W^T (library routine as a second opinion)."""
    h, W, _, _ = tiny("ff", 6, 1, 11, d=9, B=5, seed=12)
    x = np.random.default_rng(4).integers(0, 11, size=(5, 6))
    ll = oc.loglik("ff", h, W, None, None, x)
    logits = torch.einsum("nvd,bd->bnv", torch.tensor(W[:, 0]), torch.tensor(h))
    ce = torch.nn.functional.cross_entropy(logits.reshape(-1, 11), torch.tensor(x).reshape(-1),
                                           reduction="none").reshape(5, 6).sum(1)
    assert np.allclose(ll, -ce.numpy(), rtol=0, atol=1e-12)


def test_unembedding_orientation():
    """l[b,i,j,a] = <W[i,j,a,:], h[b,:]>: a one-hot h picks a column of W."""
    rng = np.random.default_rng(0)
    W = rng.standard_normal((2, 3, 4, 5))
    h = np.zeros((1, 5)); h[0, 2] = 1.0
    assert np.array_equal(oc.unembed_logits(h, W)[0], W[:, :, :, 2])


# ------------------------------------------------------------- marginals
@pytest.mark.parametrize("family,n,r,v", [("ff", 4, 1, 3), ("cp", 4, 3, 3), ("hmm", 4, 3, 3),
                                          ("btree", 4, 2, 3), ("btree", 8, 2, 2)])
def test_prefix_and_univariate_marginals_are_sums_of_the_joint(family, n, r, v):
    h, W, Wsum, layers = tiny(family, n, r, v, B=2, seed=20 + n + r)
    rng = np.random.default_rng(6)
    x = rng.integers(0, v, size=(2, n))
    P = oc.prefix_marginals(family, h, W, Wsum, layers, x)
    M = oc.univariate_marginals(family, h, W, Wsum, layers)
    L = oc.loglik(family, h, W, Wsum, layers, x)
    assert np.allclose(P[:, -1], L, rtol=0, atol=1e-13)
    assert np.all(np.diff(P, axis=1) <= 1e-13)           # prefixes only lose mass
    assert np.allclose(np.exp(M).sum(-1), 1.0, rtol=0, atol=1e-12)
    for b in range(2):
        phi, omega, lay = tables(family, h, W, Wsum, layers, b)
        tab = bf.joint_table(family, phi, omega, lay)
        for i in range(n):
            idx = tuple(x[b, :i + 1])
            assert abs(np.exp(P[b, i]) - tab[idx].sum()) < 1e-13
            axes = tuple(a for a in range(n) if a != i)
            assert np.allclose(np.exp(M[b, i]), tab.sum(axis=axes), rtol=0, atol=1e-13)


def test_arbitrary_subset_marginal_via_minus_one_targets():
    h, W, Wsum, layers = tiny("btree", 4, 2, 3, B=1, seed=31)
    phi, omega, lay = tables("btree", h, W, Wsum, layers, 0)
    tab = bf.joint_table("btree", phi, omega, lay)
    x = np.array([[-1, 2, -1, 0]])
    got = oc.loglik("btree", h, W, Wsum, layers, x)[0]
    assert abs(np.exp(got) - tab[:, 2, :, 0].sum()) < 1e-13


def test_invalid_target_gives_nan_and_neg_inf_is_safe():
    h, W, Wsum, layers = tiny("hmm", 3, 2, 3, B=2, seed=40)
    x = np.array([[0, 3, 1], [1, 1, 1]])
    ll = oc.loglik("hmm", h, W, Wsum, layers, x)
    assert np.isnan(ll[0]) and np.isfinite(ll[1])
    assert oc.logsumexp(np.array([-np.inf, -np.inf])) == -np.inf
    # a state that can never be entered: one column of the transition at -inf
    lay = np.array(layers, copy=True)
    lay[:, :, 1] = -np.inf
    ok = oc.loglik("hmm", h, W, Wsum, lay, np.array([[0, 1, 2], [2, 2, 2]]))
    assert np.all(np.isfinite(ok))


# ------------------------------------------------- the paper's printed figures
def test_parameter_counts_match_the_papers_table(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "param_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for fam, n, count, head_m in rows:
        n, count, head_m = int(n), int(count), int(head_m)
        r = 1 if fam == "ff" else 32
        got = oc.param_count(fam, n, r, 320)
        assert got == count
        assert round(got * 4096 / 1e6) == head_m


@pytest.mark.parametrize("family", ["hmm", "btree"])
def test_joint_consumes_exactly_the_counted_layers(family):
    """The evaluator takes exactly as many r x r layers as the count above says
    (and rejects one more or one fewer), tying the structure to the table."""
    n, r, v = 8, 2, 3
    shapes = oc.circuit_shapes(family, n, r, v)
    h, W, Wsum, layers = tiny(family, n, r, v, B=1, seed=1)
    assert layers.shape == shapes["layers"] and W.shape[:3] == shapes["phi"]
    x = np.zeros((1, n), dtype=np.int64)
    oc.loglik(family, h, W, Wsum, layers, x)
    for bad in (layers[:-1], np.concatenate([layers, layers[:1]])):
        with pytest.raises(AssertionError):
            oc.loglik(family, h, W, Wsum, bad, x)


def test_logit_memory_matches_the_papers_table(golden_dir):
    unit = {"MB": 2 ** 20, "GB": 2 ** 30, "TB": 2 ** 40}
    rows = [l.split() for l in open(os.path.join(golden_dir, "logit_memory.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for v, r, n, val, u in rows:
        size = oc.logits_bytes(8192, int(n), int(v), int(r)) / unit[u]
        assert abs(size - float(val)) <= 0.051, (v, r, n, size, val)


# ------------------------------------------- sum layers computed from the hidden state
def test_contextual_layer_logits_orientation_and_bias():
    rng = np.random.default_rng(0)
    R = rng.standard_normal((3, 2, 2, 5))
    bias = rng.standard_normal((3, 2, 2))
    h = np.zeros((2, 5)); h[0, 4] = 1.0; h[1, 1] = 2.0
    got = oc.contextual_layer_logits(h, R, bias)
    assert got.shape == (2, 3, 2, 2)
    assert np.allclose(got[0], R[..., 4] + bias, rtol=0, atol=1e-15)
    assert np.allclose(got[1], 2.0 * R[..., 1] + bias, rtol=0, atol=1e-15)
    assert np.array_equal(oc.contextual_layer_logits(h, R), oc.contextual_layer_logits(h, R, np.zeros((2, 2))))


@pytest.mark.parametrize("family", ["hmm", "btree"])
def test_zero_R_with_identity_bias_starts_as_cp(family):
    """Identity initialisation through a bias makes the deeper circuits equal to CP
    whatever the hidden state (App. HMM setup)."""
    n, r, v = 4, 3, 5
    h, W, Wsum, _ = tiny("cp", n, r, v, B=3, seed=13)
    L = n - 1 if family == "hmm" else n - 2
    R = np.zeros((L, r, r, h.shape[1]))
    bias = np.full((r, r), -np.inf); bias[np.arange(r), np.arange(r)] = 0.0
    x = np.random.default_rng(5).integers(0, v, size=(3, n))
    lay = oc.contextual_layer_logits(h, R, bias)
    assert np.allclose(oc.loglik(family, h, W, Wsum, lay, x), oc.loglik("cp", h, W, Wsum, None, x),
                       rtol=0, atol=1e-12)


@pytest.mark.parametrize("family", ["hmm", "btree"])
def test_contextual_from_h_equals_enumeration(family):
    n, r, v = 4, 2, 3
    h, W, Wsum, _ = tiny("cp", n, r, v, B=3, seed=17)
    L = n - 1 if family == "hmm" else n - 2
    rng = np.random.default_rng(2)
    R = rng.standard_normal((L, r, r, h.shape[1]))
    bias = rng.standard_normal((L, r, r))
    lay = oc.contextual_layer_logits(h, R, bias)
    x = rng.integers(0, v, size=(3, n))
    ll = oc.loglik(family, h, W, Wsum, lay, x)
    for b in range(3):
        phi, omega, _ = tables("cp", h, W, Wsum, None, b)
        # explicit softmax of this position's own logits R h_b + bias, written out here
        z = np.einsum("lkjd,d->lkj", R, h[b]) + bias
        T = np.exp(z - z.max(-1, keepdims=True)); T /= T.sum(-1, keepdims=True)
        p = bf.prob(family, phi, omega, T, tuple(x[b]))
        assert abs(ll[b] - np.log(p)) < 1e-12


def test_head_parameter_tensors_match_the_papers_head_counts(golden_dir):
    """With every sum unit parameterised from the hidden state, the head's tensors
    W [n,r,v,d], Wsum [r,d], R [L,r,r,d] hold the parameter totals the paper prints
    for d = 4096 (Tab. mtp-circuits-flops, MTP head column)."""
    rows = [l.split() for l in open(os.path.join(golden_dir, "param_counts.txt"))
            if l.strip() and not l.startswith("#")]
    for fam, n, _, head_m in rows:
        n, r, v, d = int(n), (1 if fam == "ff" else 32), 320, 4096
        L = {"ff": 0, "cp": 0, "hmm": n - 1, "btree": n - 2}[fam]
        total = n * r * v * d + (0 if fam == "ff" else r * d) + L * r * r * d
        assert round(total / 1e6) == int(head_m)
