"""BigBird-ETC: extra global tokens in front of the sequence.  TEST INFRASTRUCTURE ONLY.

Sec. 2, second construction: g_tok global tokens are ADDED to the N regular tokens.  The
adjacency matrix becomes B in {0,1}^{(g_tok+N) x (g_tok+N)} with B(i,:) = 1 and B(:,i) = 1 for
the global tokens i and B(g_tok+i, g_tok+j) = A(i, j) for the regular ones, A being the
sliding-window (+ random) graph on the N regular tokens, taken in blocks of b as in App. D.
Unlike ITC the number of global tokens need not be a multiple of the block length (App. E
uses 230, 256, 320 and 430 of them with blocks of 84 and 169 tokens), and the window and the
random blocks live on the regular tokens only.

Attention on that graph is eq. (AT) as before: masked softmax, written out densely in fp64.

Readings (the paper gives no formula beyond B): the regular part uses this package's
readings of App. D with g = 0 (clipped window, set union, entries < 0 of the random table
ignored); the random table is indexed by regular blocks; a key-padding mask removes keys for
every query, global tokens included.
"""
from __future__ import annotations

import numpy as np

from .attention import _softmax_rows
from .pattern import dense_mask


def dense_mask_etc(rand_idx_h, n_regular: int, b: int, w: int, n_global: int) -> np.ndarray:
    """bool [(n_global + n_regular)^2] matrix B of one head (Sec. 2, ETC construction)."""
    if n_global < 0 or n_regular % b != 0:
        raise ValueError("need n_global >= 0 and n_regular a multiple of b")
    n = n_global + n_regular
    B = np.zeros((n, n), dtype=bool)
    B[:n_global, :] = True                       # B(i, :) = 1 for global i
    B[:, :n_global] = True                       # B(:, i) = 1 for global i
    B[n_global:, n_global:] = dense_mask(rand_idx_h, n_regular, b, 0, w)   # B(g+i, g+j) = A(i, j)
    return B


def _masks(rand_idx, h, n_regular, b, w, n_global, key_mask_row):
    Bm = dense_mask_etc(None if rand_idx is None else rand_idx[h], n_regular, b, w, n_global)
    if key_mask_row is not None:
        Bm = Bm & (np.asarray(key_mask_row) != 0)[None, :]
    return Bm


def attn_fwd_etc(Q, K, V, rand_idx, b: int, w: int, n_global: int, scale: float, key_mask=None):
    """O [B,H,n,d], LSE [B,H,n] (fp64) with n = n_global + n_regular; the first n_global rows
    of Q, K, V are the global tokens.  rand_idx: None or [H, n_regular/b, r] over regular blocks."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Bn, H, n, d = Q.shape
    O = np.zeros((Bn, H, n, d))
    LSE = np.zeros((Bn, H, n))
    for bi in range(Bn):
        for h in range(H):
            A = _masks(rand_idx, h, n - n_global, b, w, n_global, None if key_mask is None else key_mask[bi])
            P, lse = _softmax_rows(scale * (Q[bi, h] @ K[bi, h].T), A)
            O[bi, h] = P @ V[bi, h]
            LSE[bi, h] = lse
    return O, LSE


def attn_bwd_etc(Q, K, V, dO, rand_idx, b: int, w: int, n_global: int, scale: float, key_mask=None):
    """Gradients of sum(O * dO) on the ETC graph (the calculus of the forward, as for ITC)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    Bn, H, n, d = Q.shape
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for bi in range(Bn):
        for h in range(H):
            A = _masks(rand_idx, h, n - n_global, b, w, n_global, None if key_mask is None else key_mask[bi])
            P, _ = _softmax_rows(scale * (Q[bi, h] @ K[bi, h].T), A)
            dV[bi, h] = P.T @ dO[bi, h]
            dP = dO[bi, h] @ V[bi, h].T
            D = (P * dP).sum(axis=1)
            dS = P * (dP - D[:, None])
            dQ[bi, h] = scale * (dS @ K[bi, h])
            dK[bi, h] = scale * (dS.T @ Q[bi, h])
    return dQ, dK, dV
