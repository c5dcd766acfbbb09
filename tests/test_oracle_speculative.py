"""Pins for the oracle of the verification step (Alg. 2, acceptance loop and the
adjusted distribution), no GPU.

The conditionals are checked against a dense joint table built by brute-force
latent enumeration, the accept / reject rule against hand-computed cases, and
the whole procedure against the property that defines speculative sampling:
every emitted token is distributed as the autoregressive verifier's conditional
given the tokens emitted before it."""
import itertools

import numpy as np
import pytest

from oracle import bruteforce as bf
from oracle import mtpc_oracle as oc
from oracle import philox
from oracle import speculative as sp

from test_oracle_circuits import tables, tiny

FAMS = ("ff", "cp", "hmm", "btree")


def circuit(family, n, r, v, seed):
    h, W, Wsum, layers = tiny(family, n, r, v, B=1, seed=seed)
    logphi, logw, loglayers = oc._params(family, h, W, Wsum, layers)
    return (h, W, Wsum, layers), logphi, logw, loglayers


@pytest.mark.parametrize("family", FAMS)
def test_conditionals_match_the_dense_joint_table(family):
    n, r, v = 4, 3, 3
    raw, logphi, logw, loglayers = circuit(family, n, r, v, seed=11)
    tab = bf.joint_table(family, *tables(family, *raw, 0))
    rng = np.random.default_rng(0)
    for _ in range(6):
        x = rng.integers(0, v, size=n)
        for j in range(n):
            sub = tab[tuple(x[:j])]                       # q(x_<j, X_j, ...)
            num = sub.reshape(v, -1).sum(axis=1) if j < n - 1 else sub
            want = num / num.sum()
            got = np.exp(sp.conditional_next(family, logphi[0], None if logw is None else logw[0],
                                             loglayers, x, j))
            np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("family", FAMS)
def test_conditionals_normalise_and_multiply_to_the_joint(family):
    n, r, v = 8, 4, 5
    raw, logphi, logw, loglayers = circuit(family, n, r, v, seed=5)
    x = np.random.default_rng(3).integers(0, v, size=n)
    total = 0.0
    for j in range(n):
        c = sp.conditional_next(family, logphi[0], None if logw is None else logw[0], loglayers, x, j)
        assert abs(np.exp(c).sum() - 1.0) < 1e-12
        total += c[x[j]]
    want = oc.joint(family, oc.evidence(logphi, x[None, :]), logw, loglayers)[0]
    assert abs(total - want) < 1e-10


def one_position_ff(q):
    """An FF 'circuit' over one token with distribution q (n = 1, r = 1)."""
    return np.log(np.asarray(q, dtype=np.float64))[None, None, None, :]


def test_acceptance_threshold_and_adjusted_distribution_by_hand():
    q = [0.2, 0.5, 0.3]
    p = np.array([[[0.5, 0.3, 0.2], [0.1, 0.1, 0.8]]])      # [B=1, n+1=2, v]
    logphi = one_position_ff(q)
    # drafted token 1: p/q = 0.6.  alpha = 0.59 accepts and the extra token comes from p[1]
    acc, tok, _ = sp.speculative_verify("ff", logphi, None, None, np.array([[1]]), p, np.array([[0.59, 0.15]]))
    assert (acc[0], tok[0]) == (1, 1)            # cdf of p[1] = .1 .2 1. -> u = .15 is token 1
    # alpha = 0.61 rejects; max(0, p - q) = [.3, 0, 0] -> token 0 whatever u is
    for u_last in (0.0, 0.5, 0.999):
        acc, tok, _ = sp.speculative_verify("ff", logphi, None, None, np.array([[1]]), p, np.array([[0.61, u_last]]))
        assert (acc[0], tok[0]) == (0, 0)
    # drafted token 0: p/q = 2.5 > 1 is always accepted
    acc, tok, _ = sp.speculative_verify("ff", logphi, None, None, np.array([[0]]), p, np.array([[0.9999, 0.25]]))
    assert (acc[0], tok[0]) == (1, 2)
    # two-token residual: p = [.1,.6,.3], q = [.2,.5,.3] -> m = [0,.1,0] / .1
    p2 = np.array([[[0.1, 0.6, 0.3], [1 / 3, 1 / 3, 1 / 3]]])
    acc, tok, _ = sp.speculative_verify("ff", logphi, None, None, np.array([[0]]), p2, np.array([[0.51, 0.7]]))
    assert (acc[0], tok[0]) == (0, 1)            # p/q = 0.5 < alpha
    np.testing.assert_allclose(sp.residual(np.array([0.5, 0.3, 0.2]), np.array([0.2, 0.5, 0.3])), [1, 0, 0])
    np.testing.assert_allclose(sp.residual(np.array([0.6, 0.1, 0.3]), np.array([0.2, 0.2, 0.6])), [1, 0, 0])
    np.testing.assert_allclose(sp.residual(np.array([0.5, 0.4, 0.1]), np.array([0.3, 0.2, 0.5])), [0.5, 0.5, 0])


def ar_tables(n, v, seed):
    """A tiny autoregressive verifier: T[k][prefix] = p(X_{k+1} | prefix), k = 0..n."""
    rng = np.random.default_rng(seed)
    return [rng.dirichlet(np.ones(v) * 1.5, size=(v,) * k) for k in range(n + 1)]


@pytest.mark.parametrize("family,n", [("ff", 3), ("cp", 3), ("hmm", 3), ("btree", 4)])
def test_emitted_tokens_follow_the_verifier(family, n):
    """Speculative sampling leaves the verifier's distribution unchanged: given
    the tokens emitted so far in a cycle, the next emitted one (an accepted draft
    token, the adjusted draw after a rejection, or the bonus draw) is a draw from
    p(. | those tokens).  Measured over many independent cycles of one circuit."""
    r, v, N = 3, 3, 24000
    raw, logphi, logw, loglayers = circuit(family, n, r, v, seed=21)
    T = ar_tables(n, v, seed=4)
    rng = np.random.default_rng(99)
    nl = oc.n_latents(family, n)
    phiN = np.broadcast_to(logphi, (N,) + logphi.shape[1:])
    lwN = None if logw is None else np.broadcast_to(logw, (N, logw.shape[1]))
    drafts = oc.sample_from(family, phiN, lwN, loglayers, rng.random((N, 1, n + nl)))[0][:, 0]
    p = np.empty((N, n + 1, v))
    for k in range(n + 1):
        p[:, k] = T[k][tuple(drafts[:, i] for i in range(k))] if k else T[0]
    acc, tok, _ = sp.speculative_verify(family, phiN, lwN, loglayers, drafts, p, rng.random((N, n + 1)))
    assert set(np.unique(acc)) == set(range(n + 1))           # every outcome occurs
    for k in range(n + 1):
        rows = np.nonzero(acc >= k)[0]                        # k tokens accepted before this one
        emitted = np.where(acc[rows] > k, drafts[rows, min(k, n - 1)], tok[rows])
        cond = T[k][tuple(drafts[rows, i] for i in range(k))] if k else np.broadcast_to(T[0], (len(rows), v))
        expect = cond.sum(axis=0)
        counts = np.bincount(emitted, minlength=v)
        assert np.all(np.abs(counts - expect) <= 4.5 * np.sqrt(0.25 * len(rows)) + 1), (k, counts, expect)


def test_verification_has_a_random_stream_of_its_own():
    """Drafting and verification called with the SAME seed and offset: the acceptance test of
    token s must not see the uniform that drew token s (it would then accept or reject in step
    with the draft and the emitted tokens would stop following the verifier).  The slot map
    gives verification a draft index no drafting call uses; checked on the words themselves and
    on the property that defines speculative sampling, Philox-driven end to end."""
    n, r, v, N = 3, 3, 3, 24000
    ud = philox.uniforms(N, 2, n + 1, seed=6, offset=2)
    uv = philox.verify_uniforms(N, n + 1, seed=6, offset=2)
    assert uv.shape == (N, n + 1) and np.all((uv >= 0) & (uv < 1))
    assert not np.any(np.all(uv == ud[:, 0], axis=1)) and not np.any(np.all(uv == ud[:, 1], axis=1))
    assert abs(np.corrcoef(uv[:, 0], ud[:, 0, 0])[0, 1]) < 0.03
    raw, logphi, logw, loglayers = circuit("cp", n, r, v, seed=21)
    T = ar_tables(n, v, seed=4)
    phiN = np.broadcast_to(logphi, (N,) + logphi.shape[1:])
    lwN = np.broadcast_to(logw, (N, logw.shape[1]))
    drafts = oc.sample_from("cp", phiN, lwN, None, ud[:, :1])[0][:, 0]
    p = np.empty((N, n + 1, v))
    for k in range(n + 1):
        p[:, k] = T[k][tuple(drafts[:, i] for i in range(k))] if k else T[0]
    acc, tok, _ = sp.speculative_verify("cp", phiN, lwN, None, drafts, p, uv)
    for k in range(n + 1):
        rows = np.nonzero(acc >= k)[0]
        emitted = np.where(acc[rows] > k, drafts[rows, min(k, n - 1)], tok[rows])
        cond = T[k][tuple(drafts[rows, i] for i in range(k))] if k else np.broadcast_to(T[0], (len(rows), v))
        counts = np.bincount(emitted, minlength=v)
        assert np.all(np.abs(counts - cond.sum(axis=0)) <= 4.5 * np.sqrt(0.25 * len(rows)) + 1), (k, counts)
    # the collision this guards against does break the property: tests fed the drafting uniforms
    acc2, tok2, _ = sp.speculative_verify("cp", phiN, lwN, None, drafts, p, ud[:, 0])
    rows = np.arange(N)
    emitted = np.where(acc2 > 0, drafts[:, 0], tok2)
    counts = np.bincount(emitted, minlength=v)
    assert np.any(np.abs(counts - N * T[0]) > 4.5 * np.sqrt(0.25 * N) + 1)


@pytest.mark.parametrize("family", FAMS)
def test_verifier_equal_to_the_draft_model_accepts_every_token(family):
    n, r, v, B = 4, 3, 4, 5
    h, W, Wsum, layers = tiny(family, n, r, v, B=B, seed=8)
    logphi, logw, loglayers = oc._params(family, h, W, Wsum, layers)
    rng = np.random.default_rng(1)
    drafts = rng.integers(0, v, size=(B, n))
    p = np.empty((B, n + 1, v))
    for b in range(B):
        for j in range(n):
            p[b, j] = np.exp(sp.conditional_next(family, logphi[b], None if logw is None else logw[b],
                                                 loglayers, drafts[b], j))
        p[b, n] = rng.dirichlet(np.ones(v))
    u = rng.random((B, n + 1)) * (1 - 1e-9)
    acc, tok, _ = sp.speculative_verify(family, logphi, logw, loglayers, drafts, p, u)
    assert np.all(acc == n)
    for b in range(B):
        assert tok[b] == int(np.searchsorted(np.cumsum(p[b, n]), u[b, n], side="right"))


def test_greedy_mode_keeps_the_longest_argmax_prefix():
    n, v, B = 4, 5, 4
    h, W, Wsum, layers = tiny("cp", n, 3, v, B=B, seed=2)
    logphi, logw, loglayers = oc._params("cp", h, W, Wsum, layers)
    rng = np.random.default_rng(5)
    p = rng.dirichlet(np.ones(v), size=(B, n + 1))
    best = p.argmax(axis=-1)
    drafts = best[:, :n].copy()
    drafts[1, 2] = (drafts[1, 2] + 1) % v         # mismatch at position 2
    drafts[2, 0] = (drafts[2, 0] + 2) % v         # mismatch at once
    drafts[3, 3] = (drafts[3, 3] + 1) % v
    acc, tok, _ = sp.speculative_verify("cp", logphi, logw, loglayers, drafts, p, np.zeros((B, n + 1)), mode="greedy")
    assert list(acc) == [4, 2, 0, 3]
    assert list(tok) == [best[0, 4], best[1, 2], best[2, 0], best[3, 3]]


def test_greedy_draft_of_the_factorised_head_is_the_mode_of_the_joint():
    n, v = 4, 3
    raw, logphi, logw, loglayers = circuit("ff", n, 1, v, seed=31)
    tab = bf.joint_table("ff", *tables("ff", *raw, 0))
    drafts, lat, _ = sp.greedy_draft("ff", logphi, logw, loglayers)
    assert tuple(drafts[0]) == np.unravel_index(np.argmax(tab), tab.shape) and lat.shape == (1, 0)


@pytest.mark.parametrize("family,n", [("cp", 4), ("hmm", 4), ("btree", 4), ("btree", 8)])
def test_greedy_draft_is_ancestral_sampling_with_the_uniforms_at_the_mode(family, n):
    """Replacing a draw by its most likely outcome is the same as handing the sampler a
    uniform that falls inside that outcome's CDF interval: build those uniforms by hand,
    decision by decision, and let the (separately pinned) sampler reproduce the draft."""
    r, v = 3, 4
    raw, logphi, logw, loglayers = circuit(family, n, r, v, seed=17)
    drafts, lat, _ = sp.greedy_draft(family, logphi, logw, loglayers)
    nl = oc.n_latents(family, n)
    u = np.zeros((1, 1, n + nl))

    def mid(logp):                       # midpoint of the CDF interval of the arg max
        p = np.exp(logp)
        k = int(np.argmax(p))
        c = np.concatenate([[0.0], np.cumsum(p)])
        return k, 0.5 * (c[k] + c[k + 1])

    lay = None if loglayers is None else np.asarray(loglayers)
    if family == "cp":
        z, u[0, 0, n] = mid(logw[0])
        leaf = [z] * n
    elif family == "hmm":
        z, u[0, 0, n] = mid(logw[0])
        leaf = [z]
        for i in range(1, n):
            z, u[0, 0, n + i] = mid(lay[i - 1][z])
            leaf.append(z)
    else:
        zs = [0] * (n - 1)
        zs[0], u[0, 0, n] = mid(logw[0])
        for m in range(1, n - 1):
            zs[m], u[0, 0, n + m] = mid(lay[m - 1][zs[(m - 1) // 2]])
        leaf = [zs[(n - 1 + i - 1) // 2] for i in range(n)]
    for i in range(n):
        _, u[0, 0, i] = mid(logphi[0, i, leaf[i]])
    d2, l2 = oc.sample_from(family, logphi, logw, loglayers, u)
    assert np.array_equal(d2[0, 0], drafts[0]) and np.array_equal(l2[0, 0], lat[0])

