"""CPU oracle for the MtPC head: TEST INFRASTRUCTURE, not a product path.

A plain, slow, float64 NumPy statement of what the head computes, written from
the paper's definitions.  Only tests, the smoke check and the bench's
``cpu_baseline`` leg may import it; it shares no code with the HIP library.

Notation (Sec. 2, 3.2, 3.3): B positions, hidden size d, window n, r units per
layer, vocabulary v.  ``h`` [B,d] is the hidden state e_t, ``W`` [n,r,v,d] the
unembedding tensor, ``Wsum`` [r,d] the slice of the sum-unit tensor R that
produces the root mixture / initial-state weights, ``layers`` the pre-softmax
logits of the remaining r x r sum layers.

Parity status: every function below is pinned by tests/test_oracle_*.py
(brute-force normalisation, latent enumeration straight from Eqs. FF/CP/HMM/BTree,
the equivalences the paper states, the parameter counts of Tab. mtp-circuits-flops,
Philox known answers).  Nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from .philox import uniforms as philox_uniforms

NEG_INF = -np.inf


# ---------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------
def logsumexp(x: np.ndarray, axis: int = -1) -> np.ndarray:
    """log sum exp along ``axis``; an all -inf slice gives -inf (never NaN)."""
    x = np.asarray(x, dtype=np.float64)
    m = np.max(x, axis=axis, keepdims=True)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        s = np.log(np.sum(np.exp(x - m_safe), axis=axis, keepdims=True))
    return np.squeeze(s + m_safe, axis=axis)


def log_softmax(x: np.ndarray, axis: int = -1) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    return x - np.expand_dims(logsumexp(x, axis=axis), axis)


# ---------------------------------------------------------------------------
# parameters of the circuit from the hidden state (Sec. 3.3)
# ---------------------------------------------------------------------------
def unembed_logits(h: np.ndarray, W: np.ndarray) -> np.ndarray:
    """l[b,i,j,a] = sum_k W[i,j,a,k] h[b,k]  (the unembedding W_ij e_t, no bias)."""
    h64 = np.asarray(h, dtype=np.float64)
    n, r, v, d = W.shape
    out = np.empty((h64.shape[0], n, r, v), dtype=np.float64)
    for i in range(n):
        for j in range(r):
            out[:, i, j, :] = h64 @ np.asarray(W[i, j], dtype=np.float64).T
    return out


def input_units(h: np.ndarray, W: np.ndarray) -> np.ndarray:
    """log phi[b,i,j,:] = log softmax(W_ij e_t): categorical input units."""
    return log_softmax(unembed_logits(h, W), axis=-1)


def sum_unit(h: np.ndarray, Wsum: np.ndarray) -> np.ndarray:
    """log omega[b,:] = log softmax(R_0 e_t): root mixture / HMM initial weights."""
    s = np.asarray(h, dtype=np.float64) @ np.asarray(Wsum, dtype=np.float64).T
    return log_softmax(s, axis=-1)


def sum_layers(layer_logits: np.ndarray) -> np.ndarray:
    """Normalise r x r sum-layer logits: softmax over the LAST axis, so that every
    sum unit's weights form a convex combination (App. B.1, normalised by design)."""
    return log_softmax(np.asarray(layer_logits, dtype=np.float64), axis=-1)


def contextual_layer_logits(h: np.ndarray, R: np.ndarray, bias=None) -> np.ndarray:
    """Sum-unit parameters computed from the hidden state (Sec. 3.3): the logits
    of the sum unit (layer l, incoming state k) over its r inputs are R[l,k] e_t,
    plus an optional input-independent bias (App. HMM setup uses one to start from
    identity transitions).  R [L,r,r,d], bias [L,r,r] or [r,r] -> logits [B,L,r,r]."""
    h64 = np.asarray(h, dtype=np.float64)
    R64 = np.asarray(R, dtype=np.float64)
    L, r, r2, d = R64.shape
    out = np.empty((h64.shape[0], L, r, r2), dtype=np.float64)
    for l in range(L):
        for k in range(r):
            out[:, l, k, :] = h64 @ R64[l, k].T
    if bias is not None:
        out = out + np.asarray(bias, dtype=np.float64)
    return out


def _layer_view(loglayers: np.ndarray, count: int, B: int) -> np.ndarray:
    """Broadcast log-normalised layers to [B or 1, count, r, r].

    Accepted: [r,r] or [1,r,r] (homogeneous), [count,r,r] (one matrix per step /
    node), or the same with a leading batch axis [B,...] (contextual)."""
    a = np.asarray(loglayers, dtype=np.float64)
    if a.ndim == 2:
        a = a[None, None]
    elif a.ndim == 3:
        a = a[None]
    assert a.ndim == 4 and a.shape[0] in (1, B)
    if a.shape[1] == 1 and count != 1:
        a = np.broadcast_to(a, (a.shape[0], count) + a.shape[2:])
    assert a.shape[1] == count, (a.shape, count)
    return a


# ---------------------------------------------------------------------------
# evidence: value of each input unit at the observed token
# ---------------------------------------------------------------------------
def evidence(logphi: np.ndarray, x: np.ndarray) -> np.ndarray:
    """e[b,i,j] = log phi[b,i,j,x[b,i]]; 0 where x[b,i] == -1 (a marginalised
    variable: its normalised input units integrate to 1, App. B.1); NaN for any
    other id outside [0, v)."""
    B, n, r, v = logphi.shape
    x = np.asarray(x)
    e = np.empty((B, n, r), dtype=np.float64)
    for b in range(B):
        for i in range(n):
            t = int(x[b, i])
            if t == -1:
                e[b, i, :] = 0.0
            elif 0 <= t < v:
                e[b, i, :] = logphi[b, i, :, t]
            else:
                e[b, i, :] = np.nan
    return e


# ---------------------------------------------------------------------------
# the four joints (Eqs. FF, CP, HMM, BTree) in log space
# ---------------------------------------------------------------------------
def ff_joint(e: np.ndarray) -> np.ndarray:
    """Eq. FF: product of the n per-position categoricals."""
    assert e.shape[2] == 1
    return np.sum(e[:, :, 0], axis=1)


def cp_joint(e: np.ndarray, logw: np.ndarray) -> np.ndarray:
    """Eq. CP: sum_z q(z) prod_i q(x_i | z)."""
    return logsumexp(logw + np.sum(e, axis=1), axis=-1)


def hmm_forward(e: np.ndarray, logw: np.ndarray, logT: np.ndarray) -> np.ndarray:
    """Forward messages of Eq. HMM:
    alpha_0[j] = log q(z_1=j) + e[0,j];
    alpha_i[j'] = e[i,j'] + log sum_j exp(alpha_{i-1}[j] + log q(z_{i+1}=j' | z_i=j)).
    logT[l][j,j'] is the transition from step l to l+1, rows (previous state)
    normalised.  Returns alpha [B,n,r]."""
    B, n, r = e.shape
    T = _layer_view(logT, n - 1, B) if n > 1 else None
    alpha = np.empty((B, n, r), dtype=np.float64)
    alpha[:, 0] = logw + e[:, 0]
    for i in range(1, n):
        # [B, j, j'] = alpha[b, j] + T[b, i-1, j, j']
        alpha[:, i] = e[:, i] + logsumexp(alpha[:, i - 1][:, :, None] + T[:, i - 1], axis=1)
    return alpha


def hmm_joint(e, logw, logT) -> np.ndarray:
    return logsumexp(hmm_forward(e, logw, logT)[:, -1], axis=-1)


def btree_joint(e: np.ndarray, logw: np.ndarray, logA: np.ndarray) -> np.ndarray:
    """Eq. BTree on a perfect binary tree over n = 2^k tokens (balanced halves).

    Heap numbering: inner nodes m = 0..n-2 (root 0, children 2m+1 and 2m+2), the
    leaf of token i is heap index n-1+i.  Each inner node owns one latent; a
    non-root node m has the r x r sum layer logA[m-1][k,j] = log q(z_m=j | z_parent=k);
    the root's weights are logw.  A leaf's r input units are indexed by its
    parent's latent.  C_m[k] = log sum_j exp(logA[m-1][k,j] + C_left[j] + C_right[j])."""
    B, n, r = e.shape
    assert n >= 2 and (n & (n - 1)) == 0, "binary tree needs n a power of two >= 2"
    A = _layer_view(logA, n - 2, B) if n > 2 else None
    C = [None] * (2 * n - 1)
    for i in range(n):
        C[n - 1 + i] = e[:, i]
    for m in range(n - 2, 0, -1):
        prod = C[2 * m + 1] + C[2 * m + 2]                      # [B, j]
        C[m] = logsumexp(A[:, m - 1] + prod[:, None, :], axis=-1)   # [B, k]
    return logsumexp(logw + C[1] + C[2], axis=-1)


def joint(family: str, e, logw=None, loglayers=None) -> np.ndarray:
    if family == "ff":
        return ff_joint(e)
    if family == "cp":
        return cp_joint(e, logw)
    if family == "hmm":
        return hmm_joint(e, logw, loglayers)
    if family == "btree":
        return btree_joint(e, logw, loglayers)
    raise ValueError(family)


# ---------------------------------------------------------------------------
# end-to-end entry points mirroring the library's
# ---------------------------------------------------------------------------
def _params(family, h, W, Wsum, layers):
    logphi = input_units(h, W)
    logw = None if family == "ff" else sum_unit(h, Wsum)
    loglayers = None if layers is None else sum_layers(layers)
    return logphi, logw, loglayers


def loglik(family, h, W, Wsum, layers, targets) -> np.ndarray:
    """log q(x_1..x_n | context) per position; targets == -1 are marginalised."""
    logphi, logw, loglayers = _params(family, h, W, Wsum, layers)
    return joint(family, evidence(logphi, targets), logw, loglayers)


def prefix_marginals_from(family, logphi, logw, loglayers, targets) -> np.ndarray:
    """P[b,i] = log q(x_1..x_{i+1}): the joint with every later variable summed
    out (Alg. 2, prefix marginals), i.e. the circuit evaluated with those input
    units replaced by 1."""
    B, n = targets.shape
    out = np.empty((B, n), dtype=np.float64)
    for i in range(n):
        x = np.array(targets, dtype=np.int64, copy=True)
        x[:, i + 1:] = -1
        out[:, i] = joint(family, evidence(logphi, x), logw, loglayers)
    return out


def prefix_marginals(family, h, W, Wsum, layers, targets) -> np.ndarray:
    logphi, logw, loglayers = _params(family, h, W, Wsum, layers)
    return prefix_marginals_from(family, logphi, logw, loglayers, targets)


def univariate_marginals(family, h, W, Wsum, layers) -> np.ndarray:
    """M[b,i,a] = log q(x_{i+1} = a): every other variable summed out."""
    logphi, logw, loglayers = _params(family, h, W, Wsum, layers)
    B, n, r, v = logphi.shape
    out = np.empty((B, n, v), dtype=np.float64)
    for i in range(n):
        for a in range(v):
            x = np.full((B, n), -1, dtype=np.int64)
            x[:, i] = a
            out[:, i, a] = joint(family, evidence(logphi, x), logw, loglayers)
    return out


# ---------------------------------------------------------------------------
# ancestral sampling (Alg. 1)
# ---------------------------------------------------------------------------
def n_latents(family: str, n: int) -> int:
    return {"ff": 0, "cp": 1, "hmm": n, "btree": n - 1}[family]


def categorical_draw(logp: np.ndarray, u: float) -> int:
    """Inverse-CDF draw: the smallest k with u < p_0 + ... + p_k, the partial sums
    taken in ascending index order in float64; if rounding leaves no such k, the
    largest k with p_k > 0."""
    p = np.exp(np.asarray(logp, dtype=np.float64))
    acc = 0.0
    for k in range(p.shape[0]):
        acc += p[k]
        if u < acc:
            return k
    pos = np.nonzero(p > 0)[0]
    return int(pos[-1])


def cdf_boundary_distance(logp: np.ndarray, u: float) -> float:
    """min_k |u - cdf[k]|: how close the uniform is to a decision boundary."""
    c = np.cumsum(np.exp(np.asarray(logp, dtype=np.float64)))
    return float(np.min(np.abs(c - u)))


def sample_from(family, logphi, logw, loglayers, u, with_margin=False):
    """Top-down traversal of the circuit (Alg. 1): at every sum unit pick ONE
    input with probability equal to its weight, at a product follow all inputs,
    at an input unit draw the token.  ``u`` [B,S,n+n_lat] are the uniforms:
    slot i drives token i, slot n+l drives latent l (CP: l=0 the mixture
    component; HMM: l=i the state z_i; BTree: l=m the latent of inner node m).

    Returns drafts [B,S,n] int32, latents [B,S,n_lat] int32 and, if asked, the
    smallest |u - cdf| met by any draw of each draft [B,S]."""
    B, n, r, v = logphi.shape
    S = u.shape[1]
    nl = n_latents(family, n)
    assert u.shape == (B, S, n + nl)
    drafts = np.empty((B, S, n), dtype=np.int32)
    lat = np.empty((B, S, nl), dtype=np.int32)
    margin = np.full((B, S), np.inf)
    if family == "hmm" and n > 1:
        T = _layer_view(loglayers, n - 1, B)
    if family == "btree" and n > 2:
        A = _layer_view(loglayers, n - 2, B)

    def draw(logp, uu, b, s):
        if with_margin:
            margin[b, s] = min(margin[b, s], cdf_boundary_distance(logp, uu))
        return categorical_draw(logp, uu)

    for b in range(B):
        for s in range(S):
            leaf_state = [0] * n
            if family == "cp":
                z = draw(logw[b], u[b, s, n], b, s)
                lat[b, s, 0] = z
                leaf_state = [z] * n
            elif family == "hmm":
                z = draw(logw[b], u[b, s, n], b, s)
                lat[b, s, 0] = z
                leaf_state[0] = z
                for i in range(1, n):
                    Tb = T[b if T.shape[0] > 1 else 0, i - 1]
                    z = draw(Tb[z], u[b, s, n + i], b, s)
                    lat[b, s, i] = z
                    leaf_state[i] = z
            elif family == "btree":
                zs = [0] * (n - 1)
                zs[0] = draw(logw[b], u[b, s, n], b, s)
                for m in range(1, n - 1):
                    Ab = A[b if A.shape[0] > 1 else 0, m - 1]
                    zs[m] = draw(Ab[zs[(m - 1) // 2]], u[b, s, n + m], b, s)
                lat[b, s, :] = zs
                for i in range(n):
                    leaf_state[i] = zs[(n - 1 + i - 1) // 2]
            for i in range(n):
                drafts[b, s, i] = draw(logphi[b, i, leaf_state[i]], u[b, s, i], b, s)
    if with_margin:
        return drafts, lat, margin
    return drafts, lat


def sample(family, h, W, Wsum, layers, S, seed, offset=0, with_margin=False,
           with_prefix=False):
    """Draft S windows per position with Philox-driven uniforms (slot map above);
    optionally also the prefix log-marginals of each draft [B,S,n]."""
    logphi, logw, loglayers = _params(family, h, W, Wsum, layers)
    B, n = logphi.shape[0], logphi.shape[1]
    u = philox_uniforms(B, S, n + n_latents(family, n), seed, offset)
    res = sample_from(family, logphi, logw, loglayers, u, with_margin=with_margin)
    if with_prefix:
        pl = np.empty((B, S, n), dtype=np.float64)
        for s in range(S):
            pl[:, s] = prefix_marginals_from(family, logphi, logw, loglayers, res[0][:, s])
        res = res + (pl,)
    return res


# ---------------------------------------------------------------------------
# bookkeeping pinned by the paper's tables
# ---------------------------------------------------------------------------
def circuit_shapes(family: str, n: int, r: int, v: int) -> dict:
    """Shapes of the per-position circuit parameters in the paper's fully
    contextual variant: input units [n,r,v], root/initial weights [r], and the
    r x r sum layers (HMM: n-1 transitions; BTree: n-2 non-root inner nodes)."""
    if family == "ff":
        return {"phi": (n, 1, v)}
    if family == "cp":
        return {"phi": (n, r, v), "omega": (r,)}
    if family == "hmm":
        return {"phi": (n, r, v), "omega": (r,), "layers": (n - 1, r, r)}
    if family == "btree":
        return {"phi": (n, r, v), "omega": (r,), "layers": (n - 2, r, r)}
    raise ValueError(family)


def param_count(family: str, n: int, r: int, v: int) -> int:
    return int(sum(int(np.prod(s)) for s in circuit_shapes(family, n, r, v).values()))


def logits_bytes(s: int, n: int, v: int, r: int, itemsize: int = 4) -> int:
    """Size of the s x n x v x r logits tensor (App. memory bottleneck)."""
    return s * n * v * r * itemsize
