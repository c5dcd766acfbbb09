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


@pytest.mark.parametrize("family,n,r,v", [("cp", 2, 3, 3), ("hmm", 3, 2, 2), ("btree", 4, 2, 2), ("ff", 3, 1, 2)])
def test_sample_frequencies_follow_the_joint(family, n, r, v):
    """Chi-square of many drafts of one position against the brute-forced joint."""
    h, W, Wsum, layers = tiny(family, n, r, v, B=1, seed=50 + n)
    S = 40000
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
