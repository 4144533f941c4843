"""Pins of the ETC oracle (oracle/etc.py) -- CPU only.

The ETC construction of Sec. 2 (extra global tokens in front of the N regular ones:
B(i,:) = B(:,i) = 1 for the global tokens, B(g+i, g+j) = A(i,j) otherwise) is pinned by
things other than itself:
  * where it coincides with the ITC construction -- a number of global tokens that is a
    multiple of b is the ITC pattern with that many leading global blocks; no global token
    at all is the window(+random) graph -- against the ITC oracle functions;
  * an independent per-element loop over the definition of B, with block sizes and token
    counts that are not powers of two;
  * the key counts the App. E tables imply: window length 252 = 3 x 84 and 507 = 3 x 169,
    230 / 256 / 320 / 430 global tokens, no random tokens: a regular token in the middle
    attends (global tokens + window length) keys;
  * closed forms for Q = 0, rows of the softmax summing to one, finite differences.
"""
import numpy as np
import pytest

import oracle
from oracle.etc import attn_bwd_etc, attn_fwd_etc, dense_mask_etc


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_multiple_of_block_global_tokens_is_itc_with_leading_global_blocks():
    b, g, w, r, H, N = 4, 2, 3, 2, 2, 40
    nb_reg = N // b
    n = g * b + N
    ridx_reg = oracle.make_rand_idx(H, N, b, 0, w, r, 7)                   # over regular blocks
    ridx_itc = np.full((H, n // b, r), -1, dtype=np.int32)
    ridx_itc[:, g:, :] = ridx_reg + g                                        # same blocks, ITC numbering
    for h in range(H):
        assert (dense_mask_etc(ridx_reg[h], N, b, w, g * b) ==
                oracle.dense_mask(ridx_itc[h], n, b, g, w, oracle.GLOBAL_LEADING)).all()
    Q, K, V, dO = (_rand((2, H, n, 8), s) for s in (1, 2, 3, 4))
    km = np.ones((2, n), dtype=np.uint8)
    km[1, 30:] = 0
    O1, L1 = attn_fwd_etc(Q, K, V, ridx_reg, b, w, g * b, 0.3, key_mask=km)
    O2, L2 = oracle.attn_fwd(Q, K, V, ridx_itc, b, g, w, 0.3, key_mask=km, global_mode=oracle.GLOBAL_LEADING)
    assert np.abs(O1 - O2).max() < 1e-13 and np.abs(L1 - L2).max() < 1e-13
    G1 = attn_bwd_etc(Q, K, V, dO, ridx_reg, b, w, g * b, 0.3, key_mask=km)
    G2 = oracle.attn_bwd(Q, K, V, dO, ridx_itc, b, g, w, 0.3, key_mask=km, global_mode=oracle.GLOBAL_LEADING)
    assert max(np.abs(a - c).max() for a, c in zip(G1, G2)) < 1e-13


def test_no_global_token_is_the_window_graph():
    b, w, N = 3, 5, 27
    M = dense_mask_etc(None, N, b, w, 0)
    assert (M == oracle.dense_mask(None, N, b, 0, w)).all()
    i, k = np.indices((N, N))
    assert (M == (np.abs(i // b - k // b) <= (w - 1) // 2)).all()


@pytest.mark.parametrize("b,w,n_global,nb_reg,r", [(3, 3, 5, 6, 0), (5, 3, 7, 4, 1), (7, 5, 1, 5, 0), (2, 1, 3, 9, 2)])
def test_mask_and_attention_by_an_independent_loop(b, w, n_global, nb_reg, r):
    """B written out element by element from Sec. 2, then softmax attention by plain loops."""
    N = nb_reg * b
    n = n_global + N
    H = 2
    rng = np.random.default_rng(100 + b)
    ridx = None
    if r:
        ridx = np.stack([np.stack([rng.choice(nb_reg, size=r, replace=False) for _ in range(nb_reg)])
                         for _ in range(H)]).astype(np.int32)
    half = (w - 1) // 2
    Q, K, V = (_rand((1, H, n, 4), s) for s in (11, 12, 13))
    O, L = attn_fwd_etc(Q, K, V, ridx, b, w, n_global, 0.7)
    for h in range(H):
        M = dense_mask_etc(None if ridx is None else ridx[h], N, b, w, n_global)
        for i in range(n):
            keys = []
            for k in range(n):
                if i < n_global or k < n_global:
                    att = True
                else:
                    ji, jk = (i - n_global) // b, (k - n_global) // b
                    att = abs(ji - jk) <= half or (ridx is not None and jk in [int(x) for x in ridx[h, ji]])
                assert M[i, k] == att, (h, i, k)
                if att:
                    keys.append(k)
            s = np.array([0.7 * sum(Q[0, h, i, c] * K[0, h, k, c] for c in range(4)) for k in keys])
            e = np.exp(s - s.max())
            want = sum((e[t] / e.sum()) * V[0, h, k] for t, k in enumerate(keys))
            assert np.abs(O[0, h, i] - want).max() < 1e-12
            assert abs(L[0, h, i] - (s.max() + np.log(e.sum()))) < 1e-12


@pytest.mark.parametrize("b,window_len,n_global", [(84, 252, 256), (84, 252, 230), (84, 252, 320), (84, 252, 430),
                                                   (169, 507, 256), (169, 507, 430)])
def test_key_counts_at_the_sizes_of_the_etc_tables(b, window_len, n_global):
    """App. E: ETC base uses blocks of 84 tokens with a window of 252 = 3 blocks, the large
    model blocks of 169 with a window of 507; 230-430 global tokens; no random tokens."""
    w = window_len // b
    assert w * b == window_len and w == 3
    nb_reg = 12
    M = dense_mask_etc(None, nb_reg * b, b, w, n_global)
    n = n_global + nb_reg * b
    rows = M.sum(axis=1)
    assert (rows[:n_global] == n).all()                                        # global tokens see everything
    assert (M[:, :n_global].sum(axis=0) == n).all()                            # and are seen by everything
    mid = n_global + 5 * b + b // 2
    assert rows[mid] == n_global + window_len                                  # regular token, middle block
    assert rows[n_global] == n_global + 2 * b and rows[-1] == n_global + 2 * b  # first / last block: clipped window
    assert int(M.sum()) == 2 * n_global * n - n_global ** 2 + b * b * (3 * nb_reg - 2)


def test_zero_queries_closed_form_rows_sum_to_one_and_finite_differences():
    b, w, n_global, nb_reg = 4, 3, 6, 5
    N = nb_reg * b
    n = n_global + N
    H = 1
    K, V = _rand((1, H, n, 5), 21), _rand((1, H, n, 5), 22)
    km = np.ones((1, n), dtype=np.uint8)
    km[0, 2] = 0          # a padded global token
    km[0, n - 3:] = 0     # padded regular tokens
    O, L = attn_fwd_etc(np.zeros_like(K), K, V, None, b, w, n_global, 1.0, key_mask=km)
    M = dense_mask_etc(None, N, b, w, n_global) & (km[0] != 0)[None, :]
    for i in range(n):
        assert abs(L[0, 0, i] - np.log(M[i].sum())) < 1e-12
        assert np.abs(O[0, 0, i] - V[0, 0][M[i]].mean(axis=0)).max() < 1e-12
    # V = 1 everywhere: O = row sums of the softmax = 1
    Q = _rand((1, H, n, 5), 23)
    O1, _ = attn_fwd_etc(Q, K, np.ones_like(V), None, b, w, n_global, 0.5, key_mask=km)
    assert np.abs(O1 - 1.0).max() < 1e-12
    # gradients against central differences of sum(O * dO)
    dO = _rand((1, H, n, 5), 24)
    dQ, dK, dV = attn_bwd_etc(Q, K, V, dO, None, b, w, n_global, 0.5, key_mask=km)
    f = lambda q, k, v: float((attn_fwd_etc(q, k, v, None, b, w, n_global, 0.5, key_mask=km)[0] * dO).sum())
    rng = np.random.default_rng(5)
    eps = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(12):
            idx = (0, 0, int(rng.integers(n)), int(rng.integers(5)))
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (f(*args_p) - f(*args_m)) / (2 * eps)
            assert abs(fd - G[idx]) < 1e-6 * max(1.0, abs(fd)), (name, idx, fd, G[idx])
    assert (dK[0, 0, 2] == 0).all() and (dV[0, 0, n - 3:] == 0).all()      # padded keys get no gradient
