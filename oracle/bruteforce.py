"""Brute-force evaluators used to pin the oracle (TEST INFRASTRUCTURE).

Everything here works in the LINEAR domain on explicit probability tables and
enumerates: all latent assignments of one window (straight from the displayed
Eqs. FF / CP / HMM / BTree), or all v^n windows.  Deliberately different in
style from mtpc_oracle.py (no log-space recursions, no message passing) so that a
slip in one is unlikely to be mirrored in the other.  Only for tiny n, r, v.

Inputs for one position: phi[n][r][v] (rows sum to 1), omega[r], and
layers[L][r][r] with rows summing to 1.
"""
from __future__ import annotations

import itertools

import numpy as np


def ff_prob(phi, x):
    """Eq. FF."""
    p = 1.0
    for i, xi in enumerate(x):
        p *= phi[i][0][xi]
    return p


def cp_prob(phi, omega, x):
    """Eq. CP: sum over the single latent z."""
    total = 0.0
    for z in range(len(omega)):
        term = omega[z]
        for i, xi in enumerate(x):
            term *= phi[i][z][xi]
        total += term
    return total


def hmm_prob(phi, omega, trans, x):
    """Eq. HMM: sum over all r^n state sequences z_1..z_n of
    q(z_1) q(x_1|z_1) prod_{i>=2} q(z_i|z_{i-1}) q(x_i|z_i)."""
    n = len(x)
    r = len(omega)
    total = 0.0
    for zs in itertools.product(range(r), repeat=n):
        term = omega[zs[0]] * phi[0][zs[0]][x[0]]
        for i in range(1, n):
            term *= trans[i - 1][zs[i - 1]][zs[i]] * phi[i][zs[i]][x[i]]
        total += term
    return total


def _btree_rec(phi, layers, x, lo, hi, node, z_parent, r):
    """q(x_lo..x_{hi-1} | latent of the parent node = z_parent) for the subtree
    rooted at heap node ``node`` (recursive reading of Eq. BTree: one sum unit
    with weights q(z_h | z_l), then the product of the two halves)."""
    if hi - lo == 1:
        return phi[lo][z_parent][x[lo]]            # base case: layer of input units
    mid = (lo + hi) // 2
    total = 0.0
    for z in range(r):
        w = layers[node - 1][z_parent][z]
        total += (w * _btree_rec(phi, layers, x, lo, mid, 2 * node + 1, z, r)
                    * _btree_rec(phi, layers, x, mid, hi, 2 * node + 2, z, r))
    return total


def btree_prob(phi, omega, layers, x):
    """Eq. BTree applied recursively from the root (whose weights are omega)."""
    n = len(x)
    r = len(omega)
    mid = n // 2
    total = 0.0
    for z in range(r):
        left = _btree_rec(phi, layers, x, 0, mid, 1, z, r)
        right = _btree_rec(phi, layers, x, mid, n, 2, z, r)
        total += omega[z] * left * right
    return total


def prob(family, phi, omega, layers, x):
    if family == "ff":
        return ff_prob(phi, x)
    if family == "cp":
        return cp_prob(phi, omega, x)
    if family == "hmm":
        return hmm_prob(phi, omega, layers, x)
    if family == "btree":
        return btree_prob(phi, omega, layers, x)
    raise ValueError(family)


def joint_table(family, phi, omega, layers):
    """Dense tensor of q over all v^n windows (the object of Eq. n-gram-prob)."""
    n = len(phi)
    v = len(phi[0][0])
    tab = np.zeros((v,) * n, dtype=np.float64)
    for x in itertools.product(range(v), repeat=n):
        tab[x] = prob(family, phi, omega, layers, x)
    return tab
