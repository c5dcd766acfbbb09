"""Pins for the oracle's ancestral sampler (Alg. 1) - no GPU."""
import itertools

import numpy as np
import pytest
from scipy import stats

from oracle import bruteforce as bf
from oracle import mtpc_oracle as oc
from oracle import philox

from test_oracle_circuits import tables, tiny


def test_categorical_draw_rule():
    logp = np.log(np.array([0.0, 0.25, 0.0, 0.5, 0.25, 0.0]))
    assert oc.categorical_draw(logp, 0.0) == 1          # zero-mass token never drawn
    assert oc.categorical_draw(logp, 0.2499999) == 1
    assert oc.categorical_draw(logp, 0.25) == 3         # strict u < cdf
    assert oc.categorical_draw(logp, 0.75) == 4
    assert oc.categorical_draw(logp, 0.9999999) == 4
    # rounding leaves the total below u: fall back to the last positive entry
    short = np.log(np.array([0.3, 0.3, 0.3, 0.0]))
    assert oc.categorical_draw(short, 0.95) == 2
    assert abs(oc.cdf_boundary_distance(logp, 0.26) - 0.01) < 1e-12


def test_draw_agrees_with_searchsorted_on_the_cdf():
    rng = np.random.default_rng(0)
    for _ in range(200):
        p = rng.dirichlet(np.ones(17))
        u = rng.random()
        assert oc.categorical_draw(np.log(p), u) == int(np.searchsorted(np.cumsum(p), u, side="right"))


def test_ff_sampler_is_n_independent_inverse_cdf_draws():
    h, W, _, _ = tiny("ff", 5, 1, 9, B=3, seed=1)
    drafts, lat = oc.sample("ff", h, W, None, None, S=4, seed=5, offset=2)
    assert lat.shape == (3, 4, 0)
    u = philox.uniforms(3, 4, 5, seed=5, offset=2)
    for b in range(3):
        phi, _, _ = tables("ff", h, W, None, None, b)
        for s in range(4):
            for i in range(5):
                assert drafts[b, s, i] == int(np.searchsorted(np.cumsum(phi[i, 0]), u[b, s, i], side="right"))


def test_slot_map_and_tree_wiring_by_hand():
    """Re-derive one BTree and one HMM draft by hand from the uniforms."""
    n, r, v = 4, 3, 5
    for fam in ("btree", "hmm"):
        h, W, Wsum, layers = tiny(fam, n, r, v, B=2, seed=3)
        drafts, lat = oc.sample(fam, h, W, Wsum, layers, S=2, seed=9)
        nl = oc.n_latents(fam, n)
        u = philox.uniforms(2, 2, n + nl, seed=9)
        for b in range(2):
            phi, omega, lay = tables(fam, h, W, Wsum, layers, b)
            pick = lambda p, uu: int(np.searchsorted(np.cumsum(p), uu, side="right"))
            for s in range(2):
                if fam == "btree":
                    z0 = pick(omega, u[b, s, n + 0])
                    z1 = pick(lay[0][z0], u[b, s, n + 1])     # node 1 = left child of root
                    z2 = pick(lay[1][z0], u[b, s, n + 2])     # node 2 = right child
                    assert list(lat[b, s]) == [z0, z1, z2]
                    states = [z1, z1, z2, z2]
                else:
                    z = [pick(omega, u[b, s, n])]
                    for i in range(1, n):
                        z.append(pick(lay[i - 1][z[-1]], u[b, s, n + i]))
                    assert list(lat[b, s]) == z
                    states = z
                for i in range(n):
                    assert drafts[b, s, i] == pick(phi[i, states[i]], u[b, s, i])


def test_tree_wiring_of_eight_leaves_in_literals():
    """One binary tree over 8 tokens (Eq. BTree, Alg. 1), every parent written out as a literal:
    inner nodes 0..6 in heap order, node 0 the root; nodes 1, 2 hang under 0, nodes 3, 4 under 1,
    nodes 5, 6 under 2; tokens 0, 1 are read from the input units selected by node 3's latent,
    tokens 2, 3 by node 4's, tokens 4, 5 by node 5's, tokens 6, 7 by node 6's.  Layer m-1 belongs
    to node m and its row is chosen by the parent's latent; the uniform of node m sits in slot
    n + m, the uniform of token i in slot i."""
    n, r, v = 8, 3, 4
    h, W, Wsum, layers = tiny("btree", n, r, v, B=2, seed=21)
    drafts, lat = oc.sample("btree", h, W, Wsum, layers, S=40, seed=4)
    u = philox.uniforms(2, 40, 15, seed=4)
    pick = lambda p, uu: int(np.searchsorted(np.cumsum(p), uu, side="right"))
    seen = set()
    for b in range(2):
        phi, omega, lay = tables("btree", h, W, Wsum, layers, b)
        for s in range(40):
            z0 = pick(omega, u[b, s, 8])
            z1 = pick(lay[0][z0], u[b, s, 9])
            z2 = pick(lay[1][z0], u[b, s, 10])
            z3 = pick(lay[2][z1], u[b, s, 11])
            z4 = pick(lay[3][z1], u[b, s, 12])
            z5 = pick(lay[4][z2], u[b, s, 13])
            z6 = pick(lay[5][z2], u[b, s, 14])
            assert list(lat[b, s]) == [z0, z1, z2, z3, z4, z5, z6]
            assert drafts[b, s, 0] == pick(phi[0, z3], u[b, s, 0])
            assert drafts[b, s, 1] == pick(phi[1, z3], u[b, s, 1])
            assert drafts[b, s, 2] == pick(phi[2, z4], u[b, s, 2])
            assert drafts[b, s, 3] == pick(phi[3, z4], u[b, s, 3])
            assert drafts[b, s, 4] == pick(phi[4, z5], u[b, s, 4])
            assert drafts[b, s, 5] == pick(phi[5, z5], u[b, s, 5])
            assert drafts[b, s, 6] == pick(phi[6, z6], u[b, s, 6])
            assert drafts[b, s, 7] == pick(phi[7, z6], u[b, s, 7])
            seen.add((z1, z2, z3, z4, z5, z6))
    # the check has teeth only if siblings disagree somewhere (else any parent map passes)
    assert any(t[0] != t[1] for t in seen) and any(t[2] != t[3] or t[4] != t[5] for t in seen)


def test_tree_of_sixteen_leaves_reads_its_leaves_from_the_last_level():
    """n = 16: token i is drawn from the unit selected by inner node 7 + i // 2 (the eight nodes of
    the last inner level, left to right), and node m >= 1 draws from the row of its layer picked
    by node (m - 1) // 2 - checked against tables, with the level structure spelled out."""
    n, r, v = 16, 2, 3
    h, W, Wsum, layers = tiny("btree", n, r, v, B=1, seed=33)
    drafts, lat = oc.sample("btree", h, W, Wsum, layers, S=60, seed=2)
    u = philox.uniforms(1, 60, 31, seed=2)
    phi, omega, lay = tables("btree", h, W, Wsum, layers, 0)
    pick = lambda p, uu: int(np.searchsorted(np.cumsum(p), uu, side="right"))
    parent = {1: 0, 2: 0, 3: 1, 4: 1, 5: 2, 6: 2, 7: 3, 8: 3, 9: 4, 10: 4, 11: 5, 12: 5, 13: 6, 14: 6}
    leaf_node = [7, 7, 8, 8, 9, 9, 10, 10, 11, 11, 12, 12, 13, 13, 14, 14]
    for s in range(60):
        z = {0: pick(omega, u[0, s, 16])}
        for m in range(1, 15):
            z[m] = pick(lay[m - 1][z[parent[m]]], u[0, s, 16 + m])
        assert list(lat[0, s]) == [z[m] for m in range(15)]
        for i in range(16):
            assert drafts[0, s, i] == pick(phi[i, z[leaf_node[i]]], u[0, s, i])


@pytest.mark.parametrize("family,n,r,v", [("cp", 2, 3, 3), ("hmm", 3, 2, 2), ("btree", 4, 2, 2), ("ff", 3, 1, 2),
                                          ("btree", 8, 2, 2), ("btree", 8, 3, 2)])
def test_sample_frequencies_follow_the_joint(family, n, r, v):
    """Chi-square of many drafts of one position against the brute-forced joint (for the tree over
    8 tokens: 256 windows, which a wrong parent anywhere below the root's children would skew)."""
    h, W, Wsum, layers = tiny(family, n, r, v, B=1, seed=50 + n)
    S = 60000 if n == 8 else 40000
    drafts, lat = oc.sample(family, h, W, Wsum, layers, S=S, seed=77)
    phi, omega, lay = tables(family, h, W, Wsum, layers, 0)
    tab = bf.joint_table(family, phi, omega, lay)
    counts = np.zeros_like(tab)
    for x in drafts[0]:
        counts[tuple(x)] += 1
    chi2 = ((counts - S * tab) ** 2 / (S * tab)).sum()
    dof = tab.size - 1
    assert chi2 < stats.chi2.ppf(0.9999, dof), (chi2, dof)
    if family != "ff":
        f = np.bincount(lat[0, :, 0], minlength=r) / S      # root latent ~ omega
        assert np.allclose(f, omega, atol=4 * np.sqrt(0.25 / S))


def test_prefix_scores_of_drafts():
    h, W, Wsum, layers = tiny("hmm", 3, 2, 4, B=2, seed=8)
    drafts, lat, pl = oc.sample("hmm", h, W, Wsum, layers, S=3, seed=1, with_prefix=True)
    for s in range(3):
        assert np.allclose(pl[:, s], oc.prefix_marginals("hmm", h, W, Wsum, layers, drafts[:, s]))
