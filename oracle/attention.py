"""Masked softmax attention on the dense BigBird adjacency matrix, fp64.  TEST INFRASTRUCTURE ONLY.

Eq. (AT) of Sec. 2, per head, with sigma = softmax:

    out_i = softmax( scale * q_i K_{N(i)}^T ) V_{N(i)}

N(i) is read off the dense 0/1 matrix A (Sec. 2) built in `pattern.dense_mask`.
BigBird attention is exact attention on a fixed graph, so this is the definition
written out -- no blocking, no streaming softmax.  The residual `x_i +` and the
sum over heads of eq. (AT) belong to the caller: outputs are per head.

Readings where the paper is silent:
  * eq. (AT) carries no 1/sqrt(d); `scale` is an explicit argument;
  * a key-padding mask (never mentioned in the paper) removes keys for every
    query, global rows included; a row left without any key gives O = 0,
    LSE = -inf and zero gradients;
  * LSE is the natural log of the sum of exp(scale * q.k) over N(i);
  * optional (skip_padded_query_blocks): the same mask read as a query mask at block
    granularity -- a query block in which every position is padded has no neighbours at all
    (O = 0, LSE = -inf, no gradient through it), the way a caller that never reads padded
    rows would want them; blocks with at least one valid position are unchanged.
The backward pass is not in the paper; it is the calculus of the forward.
"""
from __future__ import annotations

import numpy as np

from .pattern import GLOBAL_FIRST_LAST, dense_mask


def _adjacency(rand_idx_h, n, b, g, w, global_mode, key_valid_row, skip_padded_query_blocks=False):
    A = dense_mask(rand_idx_h, n, b, g, w, global_mode)
    if key_valid_row is not None:
        valid = np.asarray(key_valid_row) != 0
        A = A & valid[None, :]
        if skip_padded_query_blocks:
            block_has_valid = valid.reshape(n // b, b).any(axis=1)
            A = A & np.repeat(block_has_valid, b)[:, None]
    return A


def _softmax_rows(S: np.ndarray, A: np.ndarray):
    """Row softmax of S restricted to A.  Returns (P, LSE); empty rows give P = 0, LSE = -inf."""
    S = np.where(A, S, -np.inf)
    m = S.max(axis=1)
    has = np.isfinite(m)
    m_safe = np.where(has, m, 0.0)
    E = np.where(A, np.exp(S - m_safe[:, None]), 0.0)
    l = E.sum(axis=1)
    with np.errstate(divide="ignore"):
        LSE = np.where(has, m_safe + np.log(np.where(has, l, 1.0)), -np.inf)
    P = E / np.where(has, l, 1.0)[:, None]
    return P, LSE


def attn_fwd(Q, K, V, rand_idx, b: int, g: int, w: int, scale: float,
             key_mask=None, global_mode: int = GLOBAL_FIRST_LAST, skip_padded_query_blocks: bool = False):
    """O [B,H,n,d] and LSE [B,H,n] in fp64 for Q, K, V [B,H,n,d] (eq. (AT), per head).

    rand_idx is [H, n/b, r]; key_mask is None or [B, n] with non-zero = valid key.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, n, d = Q.shape
    O = np.zeros((B, H, n, d))
    LSE = np.zeros((B, H, n))
    for bi in range(B):
        for h in range(H):
            A = _adjacency(rand_idx[h], n, b, g, w, global_mode,
                           None if key_mask is None else key_mask[bi], skip_padded_query_blocks)
            S = scale * (Q[bi, h] @ K[bi, h].T)
            P, lse = _softmax_rows(S, A)
            O[bi, h] = P @ V[bi, h]
            LSE[bi, h] = lse
    return O, LSE


def attn_fwd_rows(Q, K, V, rand_idx, b: int, g: int, w: int, scale: float, bi: int, h: int,
                  rows, key_mask=None, global_mode: int = GLOBAL_FIRST_LAST,
                  skip_padded_query_blocks: bool = False):
    """The same outputs for selected query rows of one (batch, head): O [len(rows), d], LSE [len(rows)].

    Used to sample large problems; each row is the definition evaluated on its own.
    """
    rows = np.asarray(rows, dtype=np.int64)
    Kf = np.asarray(K[bi, h], dtype=np.float64)
    Vf = np.asarray(V[bi, h], dtype=np.float64)
    Qf = np.asarray(Q[bi, h][rows], dtype=np.float64)
    n = Kf.shape[0]
    nb = n // b
    from .pattern import neighbour_blocks
    A = np.zeros((len(rows), n), dtype=bool)
    for t, i in enumerate(rows):
        for k in neighbour_blocks(rand_idx[h], nb, int(i) // b, g, w, global_mode):
            A[t, k * b:(k + 1) * b] = True
    if key_mask is not None:
        valid = np.asarray(key_mask[bi]) != 0
        A &= valid[None, :]
        if skip_padded_query_blocks:
            for t, i in enumerate(rows):
                j = int(i) // b
                if not valid[j * b:(j + 1) * b].any():
                    A[t, :] = False
    S = scale * (Qf @ Kf.T)
    P, lse = _softmax_rows(S, A)
    return P @ Vf, lse


def attn_bwd(Q, K, V, dO, rand_idx, b: int, g: int, w: int, scale: float,
             key_mask=None, global_mode: int = GLOBAL_FIRST_LAST, skip_padded_query_blocks: bool = False):
    """Gradients dQ, dK, dV [B,H,n,d] (fp64) of L = sum(O * dO) w.r.t. Q, K, V.

    With P the row softmax:  dV = P^T dO;  dP = dO V^T;  D_i = sum_k P_ik dP_ik;
    dS = P o (dP - D);  dQ = scale dS K;  dK = scale dS^T Q.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    B, H, n, d = Q.shape
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for bi in range(B):
        for h in range(H):
            A = _adjacency(rand_idx[h], n, b, g, w, global_mode,
                           None if key_mask is None else key_mask[bi], skip_padded_query_blocks)
            S = scale * (Q[bi, h] @ K[bi, h].T)
            P, _ = _softmax_rows(S, A)
            dV[bi, h] = P.T @ dO[bi, h]
            dP = dO[bi, h] @ V[bi, h].T
            D = (P * dP).sum(axis=1)
            dS = P * (dP - D[:, None])
            dQ[bi, h] = scale * (dS @ K[bi, h])
            dK[bi, h] = scale * (dS.T @ Q[bi, h])
    return dQ, dK, dV
