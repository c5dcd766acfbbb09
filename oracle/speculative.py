"""CPU oracle for the verification half of a speculative-decoding cycle:
TEST INFRASTRUCTURE, not a product path (same rules as mtpc_oracle.py).

States the outcome of the accept / reject part of Alg. 2 (speculative sampling with a
circuit as the draft model) in float64 - all acceptance tests of a row at once, the
first failed one decides - and the greedy variant the paper evaluates next to it (Sec. 3.4: a draft token survives iff it is the verifier's
argmax).  The conditional of the draft model is taken from its definition, a
ratio of two prefix marginals, for every candidate token: no message passing,
no reuse of anything the HIP library does.

Random numbers are inputs: ``u`` [B, n+1]; slot s < n is the alpha of the s-th
acceptance test, slot n drives the single token drawn at the end.

Parity status: pinned by tests/test_oracle_speculative.py (normalisation and
chain rule of the conditionals, brute-force suffix enumeration, the
distribution-preservation property of speculative sampling measured on a tiny
autoregressive verifier, exact acceptance when verifier == draft model, the
greedy chain).  Nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from . import mtpc_oracle as oc


def conditional_next(family, logphi_b, logw_b, loglayers_b, tokens, j) -> np.ndarray:
    """log q(X_{j+1} = a | x_1..x_j) for every a (0-based position j), Alg. 2:
    q(x_1..x_j, a) / q(x_1..x_j), both prefix marginals (later positions summed out).

    logphi_b [n,r,v], logw_b [r] or None, loglayers_b [L,r,r] or None: one position's circuit."""
    n, r, v = logphi_b.shape
    e = np.zeros((v, n, r))
    for i in range(j):
        e[:, i, :] = logphi_b[i, :, tokens[i]][None, :]
    e_den = e[:1].copy()                                   # position j summed out as well
    e[:, j, :] = logphi_b[j].T                             # candidate a at position j
    lw = None if logw_b is None else np.asarray(logw_b)[None, :]
    num = oc.joint(family, e, lw, loglayers_b)
    den = oc.joint(family, e_den, lw, loglayers_b)
    return num - den[0]


def draw_linear(w: np.ndarray, u: float):
    """Inverse-CDF draw from non-negative weights w / sum(w): smallest k with
    u < cdf[k] (ascending index order), else the largest k with w[k] > 0.
    Also returns min_k |u - cdf[k]|."""
    p = np.asarray(w, dtype=np.float64)
    p = p / p.sum()
    cdf = np.cumsum(p)
    margin = float(np.min(np.abs(cdf - u)))
    hit = np.nonzero(u < cdf)[0]
    if hit.size:
        return int(hit[0]), margin
    return int(np.nonzero(p > 0)[0][-1]), margin


def residual(p_next: np.ndarray, q_next: np.ndarray):
    """Alg. 2, adjusted distribution after a rejection: max(0, p - q) / Z.
    Z == 0 only if p == q, where a rejection has probability zero; then p itself."""
    m = np.maximum(0.0, p_next - q_next)
    Z = m.sum()
    return (m / Z) if Z > 0 else p_next


def speculative_verify(family, logphi, logw, loglayers, drafts, p, u, mode="sampling"):
    """One verification per position b (the accept / reject half of Alg. 2).

    drafts [B,n] int; p [B,n+1,v] verifier probabilities p(X_{t+i} | x_{<=t+i-1})
    evaluated along the draft; u [B,n+1] uniforms.

    What the procedure defines, stated without its loop: test s passes iff
    u[b,s] <= p[b,s,x_s] / q(x_s | x_<s) (greedy: iff x_s is the argmax of p[b,s]); the number
    of accepted tokens is the length of the leading run of passed tests; the token emitted
    after them is drawn with u[b,n] from the adjusted distribution at the first failed test,
    or from p[b,n] when none failed (greedy: the argmax there).

    Returns accepted [B] (0..n), token [B], and margin [B]: the smallest distance of any
    decision that mattered for that row from its boundary (|u - p/q| of the tests up to and
    including the first failed one, |u - cdf| of the final draw; inf in greedy mode)."""
    B, n, r, v = logphi.shape
    assert drafts.shape == (B, n) and p.shape == (B, n + 1, v) and u.shape == (B, n + 1)
    rows = np.arange(B)
    p_draft = p[rows[:, None], np.arange(n)[None, :], drafts]              # p[b,s,x_s]
    if mode == "greedy":
        passed = drafts == np.argmax(p[:, :n], axis=-1)
    else:
        P = oc.prefix_marginals_from(family, logphi, logw, loglayers, drafts)
        logq = np.diff(P, axis=1, prepend=0.0)                              # log q(x_s | x_<s)
        ratio = p_draft / np.exp(logq)
        passed = u[:, :n] <= ratio
    # length of the leading run of passed tests = index of the first failed one (n if none)
    accepted = np.where(passed.all(axis=1), n, np.argmin(passed, axis=1)).astype(np.int32)
    token = np.zeros(B, dtype=np.int32)
    margin = np.full(B, np.inf)
    if mode == "greedy":
        token[:] = np.argmax(p[rows, accepted], axis=-1)
        return accepted, token, margin
    taken = np.arange(n)[None, :] <= accepted[:, None]                      # tests that were decisive
    margin = np.min(np.where(taken, np.abs(u[:, :n] - ratio), np.inf), axis=1)
    for b in range(B):
        s = int(accepted[b])
        dist = p[b, n]
        if s < n:
            lay = None
            if loglayers is not None:
                lay = loglayers[b] if loglayers.ndim == 4 else loglayers
            q_next = np.exp(conditional_next(family, logphi[b], None if logw is None else logw[b],
                                             lay, drafts[b], s))
            dist = residual(p[b, s], q_next)
        token[b], mg = draw_linear(dist, u[b, n])
        margin[b] = min(margin[b], mg)
    return accepted, token, margin


def greedy_draft(family, logphi, logw, loglayers):
    """Draft for greedy speculative decoding (Sec. 3.4): the top-down traversal of Alg. 1
    with every draw replaced by the most likely outcome (first index on ties) - each sum
    unit takes its largest weight, each selected input unit its most likely token.
    Returns drafts [B,n], latents [B,n_lat] and, per position, the smallest gap between
    the two largest probabilities met at any of its decisions."""
    B, n, r, v = logphi.shape
    nl = oc.n_latents(family, n)
    drafts = np.zeros((B, n), dtype=np.int32)
    lat = np.zeros((B, nl), dtype=np.int32)
    gap = np.full(B, np.inf)
    if family == "hmm" and n > 1:
        T = oc._layer_view(loglayers, n - 1, B)
    if family == "btree" and n > 2:
        A = oc._layer_view(loglayers, n - 2, B)

    def pick(logp, b):
        p = np.exp(np.asarray(logp, dtype=np.float64))
        k = int(np.argmax(p))
        if p.size > 1:
            top = np.sort(p)[-2:]
            gap[b] = min(gap[b], top[1] - top[0])
        return k

    for b in range(B):
        leaf_state = [0] * n
        if family == "cp":
            lat[b, 0] = pick(logw[b], b)
            leaf_state = [int(lat[b, 0])] * n
        elif family == "hmm":
            z = pick(logw[b], b)
            lat[b, 0] = leaf_state[0] = z
            for i in range(1, n):
                z = pick(T[b if T.shape[0] > 1 else 0, i - 1][z], b)
                lat[b, i] = leaf_state[i] = z
        elif family == "btree":
            zs = [0] * (n - 1)
            zs[0] = pick(logw[b], b)
            for m in range(1, n - 1):
                zs[m] = pick(A[b if A.shape[0] > 1 else 0, m - 1][zs[(m - 1) // 2]], b)
            lat[b] = zs
            leaf_state = [zs[(n - 1 + i - 1) // 2] for i in range(n)]
        for i in range(n):
            drafts[b, i] = pick(logphi[b, i, leaf_state[i]], b)
    return drafts, lat, gap

