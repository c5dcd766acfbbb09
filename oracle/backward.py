"""CPU oracle for the training step of the MtPC head: TEST INFRASTRUCTURE, not a
product path (same rules as mtpc_oracle.py).

The loss is the discounted, locally normalised negative log-likelihood of
Sec. 4.1 (Eq. cross-ent-loss and the discount L = sum_j gamma^(j-1) L_j): token j
of a window contributes -log q(x_j | x_<j) = P[j-2] - P[j-1], a difference of
prefix log-marginals of the circuit.  The forward pass is written out once more
in float64 PyTorch, from the same equations as the NumPy oracle (Eqs. FF, CP,
HMM, BTree with the conventions stated there) and the gradients are whatever
reverse-mode differentiation of that forward pass gives: no hand-derived
backward formula lives here.

Parity status: pinned by tests/test_oracle_backward.py (forward equal to the
NumPy oracle, gradients equal to central finite differences of a loss computed
with the NumPy oracle alone, the textbook softmax-minus-one-hot gradient for FF,
telescoping to the plain log-likelihood, the coefficient table by hand).
Nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np
import torch


def loss_coefficients(gamma: float, valid: np.ndarray, sequence=None) -> np.ndarray:
    """coef[b,j] such that  loss = sum_{b,j} coef[b,j] * (-log q(x_{j+1} | x_<=j))  (0-based j).

    Eq. cross-ent-loss: L_j = -(1/N) sum_i (1/V_ij) sum_t log p(...), L = sum_j gamma^(j-1) L_j.
    ``valid`` [B,n] marks the (position, window slot) pairs that carry a target;
    ``sequence`` [B] gives the training sequence i of each position (default: all
    positions belong to one sequence); V_ij counts the valid pairs of sequence i in
    slot j and N is the number of sequences."""
    valid = np.asarray(valid, dtype=bool)
    B, n = valid.shape
    seq = np.zeros(B, dtype=np.int64) if sequence is None else np.asarray(sequence, dtype=np.int64)
    ids = np.unique(seq)
    coef = np.zeros((B, n), dtype=np.float64)
    for i in ids:
        rows = seq == i
        V = valid[rows].sum(axis=0)                      # [n]
        for j in range(n):
            if V[j] > 0:
                coef[rows, j] = (gamma ** j) * valid[rows, j] / (len(ids) * V[j])
    return coef


def _joint(family, e, logw, loglayers):
    """log q of Eqs. FF / CP / HMM / BTree from evidence e [B,n,r] (log domain)."""
    B, n, r = e.shape
    if family == "ff":
        return e[:, :, 0].sum(dim=1)
    if family == "cp":
        return torch.logsumexp(logw + e.sum(dim=1), dim=-1)
    if family == "hmm":
        alpha = logw + e[:, 0]
        for i in range(1, n):
            if loglayers.dim() == 4:                                       # one set per position [B,L,prev,next]
                T = loglayers[:, i - 1 if loglayers.shape[1] > 1 else 0]
            else:
                T = loglayers[i - 1 if loglayers.shape[0] > 1 else 0][None]    # [prev, next]
            alpha = e[:, i] + torch.logsumexp(alpha[:, :, None] + T, dim=1)
        return torch.logsumexp(alpha, dim=-1)
    if family == "btree":
        C = [None] * (2 * n - 1)
        for i in range(n):
            C[n - 1 + i] = e[:, i]
        for m in range(n - 2, 0, -1):
            if loglayers.dim() == 4:
                A = loglayers[:, m - 1 if loglayers.shape[1] > 1 else 0]
            else:
                A = loglayers[m - 1 if loglayers.shape[0] > 1 else 0][None]    # [parent's latent k, own latent j]
            prod = C[2 * m + 1] + C[2 * m + 2]
            C[m] = torch.logsumexp(A + prod[:, None, :], dim=-1)
        return torch.logsumexp(logw + C[1] + C[2], dim=-1)
    raise ValueError(family)


def prefix_marginals_torch(family, h, W, Wsum, layers, targets, R=None):
    """P[b,i] = log q(x_1..x_{i+1}) as a differentiable float64 tensor (Sec. 3.3
    parameterisation, App. B.1 marginalisation: later input units become 1).
    With R [L,r,r,d] the layer logits of position b are R h[b] + layers (Sec. 3.3: the
    sum-unit parameters are computed from the hidden state; ``layers`` is then a bias)."""
    B, n = targets.shape
    logits = torch.einsum("nrvd,bd->bnrv", W, h)
    logphi = torch.log_softmax(logits, dim=-1)
    tt = torch.as_tensor(targets, dtype=torch.int64)
    idx = tt.clamp(min=0)[:, :, None, None].expand(B, n, W.shape[1], 1)
    e = torch.gather(logphi, 3, idx)[..., 0]                               # [B,n,r]
    e = e * (tt != -1)[:, :, None]          # a target of -1 is summed out: its input units are 1 (App. B.1)
    logw = None if Wsum is None else torch.log_softmax(h @ Wsum.T, dim=-1)
    if R is not None:
        lay = torch.einsum("lzyd,bd->blzy", R, h)
        if layers is not None:
            lay = lay + layers[None]
        loglayers = torch.log_softmax(lay, dim=-1)
    else:
        loglayers = None if layers is None else torch.log_softmax(layers, dim=-1)
    cols = []
    for i in range(n):
        mask = torch.zeros(n, dtype=torch.float64)
        mask[: i + 1] = 1.0
        cols.append(_joint(family, e * mask[None, :, None], logw, loglayers))
    return torch.stack(cols, dim=1)


def loss_and_gradients(family, h, W, Wsum, layers, targets, coef, R=None):
    """Per-position loss  loss[b] = sum_j coef[b,j] * (P[b,j-1] - P[b,j])  (P[b,-1] = 0)
    and the gradients of sum_b loss[b] with respect to h, W, Wsum, the layer logits
    (or, with R, the bias) and R."""
    t = lambda a: None if a is None else torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    h_t, W_t, Ws_t, L_t, R_t = t(h), t(W), t(Wsum), t(layers), t(R)
    P = prefix_marginals_torch(family, h_t, W_t, Ws_t, L_t, np.asarray(targets), R_t)
    prev = torch.cat([torch.zeros(P.shape[0], 1, dtype=torch.float64), P[:, :-1]], dim=1)
    loss_b = (torch.as_tensor(np.asarray(coef, dtype=np.float64)) * (prev - P)).sum(dim=1)
    loss_b.sum().backward()
    g = lambda a: None if a is None else a.grad.numpy()
    return {"loss": loss_b.detach().numpy(), "P": P.detach().numpy(), "dh": g(h_t), "dW": g(W_t),
            "dWsum": g(Ws_t), "dlayers": g(L_t), "dR": g(R_t)}
