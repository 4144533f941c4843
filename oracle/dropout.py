"""Attention dropout on the BigBird graph, fp64.  TEST INFRASTRUCTURE ONLY.

The paper trains with "attention dropout 0.1" (hyper-parameter tables of App. E.1) and says no
more about it; the reading taken here is the usual one for Transformer encoders: after the row
softmax of eq. (AT), every attended probability P_ij is kept with probability 1 - p and scaled by
1 / (1 - p), independently per (batch, head, query i, key j):

    O_i = sum_j  M_ij / (1 - p) * P_ij * V_j,        M_ij in {0, 1}.

LSE is that of the undropped softmax.  With the mask fixed, the backward pass is the calculus of
this forward:  dV = (M o P / (1-p))^T dO;  dP = M / (1-p) o (dO V^T);  D_i = sum_j P_ij dP_ij
(= sum_c dO_ic O_ic);  dS = P o (dP - D);  dQ = scale dS K;  dK = scale dS^T Q.

The mask is a pure function of (seed, batch*H + head, i, j), so that a forward and a backward
call, and any tiling of either, see the same mask.  Generator (counter based, 32-bit integers):

    mix(x):   x ^= x >> 16;  x *= 0x7feb352d;  x ^= x >> 15;  x *= 0x846ca68b;  x ^= x >> 16
              (a published two-multiplication integer finaliser, "lowbias32")
    row key   rk(i)    = mix(seed_lo ^ mix(seed_hi ^ (bh * n + i)))
    word      w(i, j)  = mix(rk(i) ^ ((j >> 1) * 0x9E3779B9))          (all arithmetic mod 2^32)
    number    u(i, j)  = 15 bits of w: bits 0..14 for even j, bits 16..30 for odd j
    keep      M_ij     = [ u(i, j) >= T ],   T = round(p * 32768)

so the drop probability realised is T / 32768 (0.100006 for p = 0.1) and the kept entries are
scaled by 32768 / (32768 - T).  p = 0 keeps everything and reproduces attn_fwd / attn_bwd.

This definition is this library's, not the paper's (the paper gives none): what is pinned in
tests/test_oracle_dropout_pins.py is the arithmetic around it (p = 0, closed form for Q = 0 by
explicit loops, unbiasedness over seeds, finite differences with the mask fixed) and the
statistics of the generator (keep rate, independence of neighbours, of rows, of seeds), plus an
integer-by-integer scalar re-evaluation.  Agreement with the authors' dropout stream is
"parity unpinned": nothing in the paper fixes it.
"""
from __future__ import annotations

import numpy as np

from .attention import _adjacency, _softmax_rows
from .pattern import GLOBAL_FIRST_LAST

_M1 = np.uint32(0x7FEB352D)
_M2 = np.uint32(0x846CA68B)
_GOLD = np.uint32(0x9E3779B9)


def dropout_threshold(p: float) -> int:
    """T = round(p * 32768); p must lie in [0, 1) and T < 32768."""
    if not (0.0 <= p < 1.0):
        raise ValueError("dropout probability must be in [0, 1)")
    T = int(np.floor(p * 32768.0 + 0.5))
    if T >= 32768:
        raise ValueError("dropout probability too close to 1")
    return T


def dropout_scale(p: float) -> float:
    """1 / (1 - p_eff) for the probability actually realised, p_eff = T / 32768."""
    return 32768.0 / (32768.0 - dropout_threshold(p))


def mix32(x):
    """The integer finaliser above on uint32 arrays (wrap-around arithmetic)."""
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= _M1
    x ^= x >> np.uint32(15)
    x *= _M2
    x ^= x >> np.uint32(16)
    return x


def keep_mask(seed: int, bh: int, n: int, p: float, rows=None) -> np.ndarray:
    """M [len(rows), n] (bool) of one (batch, head) slice; rows defaults to all n queries."""
    T = dropout_threshold(p)
    rows = np.arange(n, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    s_lo = np.uint32(seed & 0xFFFFFFFF)
    s_hi = np.uint32(seed >> 32)
    with np.errstate(over="ignore"):
        rowid = ((bh * n + rows) & 0xFFFFFFFF).astype(np.uint32)
        rk = mix32(s_lo ^ mix32(s_hi ^ rowid))                         # [rows]
        pair = (np.arange(n, dtype=np.int64) >> 1).astype(np.uint32) * _GOLD  # [n]
        w = mix32(rk[:, None] ^ pair[None, :])                         # [rows, n]
    odd = (np.arange(n) & 1).astype(bool)
    u = np.where(odd[None, :], (w >> np.uint32(16)) & np.uint32(0x7FFF), w & np.uint32(0x7FFF))
    return u >= np.uint32(T)


def attn_fwd_dropout(Q, K, V, rand_idx, b: int, g: int, w: int, scale: float, p: float, seed: int,
                     key_mask=None, global_mode: int = GLOBAL_FIRST_LAST, skip_padded_query_blocks: bool = False):
    """O [B,H,n,d] with attention dropout, and the undropped LSE [B,H,n]; fp64."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, n, d = Q.shape
    rs = dropout_scale(p)
    O = np.zeros((B, H, n, d))
    LSE = np.zeros((B, H, n))
    for bi in range(B):
        for h in range(H):
            A = _adjacency(rand_idx[h], n, b, g, w, global_mode,
                           None if key_mask is None else key_mask[bi], skip_padded_query_blocks)
            S = scale * (Q[bi, h] @ K[bi, h].T)
            P, lse = _softmax_rows(S, A)
            M = keep_mask(seed, bi * H + h, n, p)
            O[bi, h] = (np.where(M, P, 0.0) * rs) @ V[bi, h]
            LSE[bi, h] = lse
    return O, LSE


def attn_fwd_dropout_rows(Q, K, V, rand_idx, b: int, g: int, w: int, scale: float, p: float,
                          seed: int, bi: int, h: int, rows, key_mask=None,
                          global_mode: int = GLOBAL_FIRST_LAST):
    """The same outputs for selected query rows of one (batch, head): O [len(rows), d], LSE
    [len(rows)].  Each row is the definition evaluated on its own (for sampling large problems)."""
    from .pattern import neighbour_blocks
    rows = np.asarray(rows, dtype=np.int64)
    H = np.asarray(Q).shape[1]
    Kf = np.asarray(K[bi, h], dtype=np.float64)
    Vf = np.asarray(V[bi, h], dtype=np.float64)
    Qf = np.asarray(Q[bi, h][rows], dtype=np.float64)
    n = Kf.shape[0]
    A = np.zeros((len(rows), n), dtype=bool)
    for t, i in enumerate(rows):
        for k in neighbour_blocks(rand_idx[h], n // b, int(i) // b, g, w, global_mode):
            A[t, k * b:(k + 1) * b] = True
    if key_mask is not None:
        A &= (np.asarray(key_mask[bi]) != 0)[None, :]
    P, lse = _softmax_rows(scale * (Qf @ Kf.T), A)
    M = keep_mask(seed, bi * H + h, n, p, rows=rows)
    return (np.where(M, P, 0.0) * dropout_scale(p)) @ Vf, lse


def attn_bwd_dropout(Q, K, V, dO, rand_idx, b: int, g: int, w: int, scale: float, p: float,
                     seed: int, key_mask=None, global_mode: int = GLOBAL_FIRST_LAST, skip_padded_query_blocks: bool = False):
    """dQ, dK, dV [B,H,n,d] (fp64) of L = sum(O * dO) for the forward above, mask held fixed."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    B, H, n, d = Q.shape
    rs = dropout_scale(p)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for bi in range(B):
        for h in range(H):
            A = _adjacency(rand_idx[h], n, b, g, w, global_mode,
                           None if key_mask is None else key_mask[bi], skip_padded_query_blocks)
            S = scale * (Q[bi, h] @ K[bi, h].T)
            P, _ = _softmax_rows(S, A)
            Mr = np.where(keep_mask(seed, bi * H + h, n, p), rs, 0.0)
            dV[bi, h] = (P * Mr).T @ dO[bi, h]
            dP = Mr * (dO[bi, h] @ V[bi, h].T)
            D = (P * dP).sum(axis=1)
            dS = P * (dP - D[:, None])
            dQ[bi, h] = scale * (dS @ K[bi, h])
            dK[bi, h] = scale * (dS.T @ Q[bi, h])
    return dQ, dK, dV
