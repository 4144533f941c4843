"""Pins of the dropout oracle (oracle/dropout.py) -- CPU only.

The paper only names the rate ("attention dropout 0.1", App. E.1); the oracle's reading -- keep
each attended probability with probability 1 - p, scale the kept ones by 1 / (1 - p), LSE
unchanged, mask a fixed function of (seed, batch*H + head, i, j) -- is pinned by things other
than itself:
  * p = 0 is the undropped forward and backward;
  * the mask generator, integer by integer in plain Python, and its statistics: keep rate,
    independence of the two numbers cut from one word, of neighbouring rows, heads and seeds,
    no collision of the mixing function on a million consecutive inputs;
  * Q = 0 makes the softmax uniform: O_i = 1/((1-p)|N(i)|) * sum of the kept V_j, by explicit
    loops over the mask and the edge list;
  * the mean over seeds tends to the undropped output (the scaling makes dropout unbiased);
  * central finite differences of L = sum(O * dO) with the mask held fixed;
  * D_i = sum_j P_ij dP_ij equals sum_c dO_ic O_ic (what a kernel computes instead).
"""
import numpy as np
import pytest

import oracle
from oracle.dropout import (attn_bwd_dropout, attn_fwd_dropout, dropout_scale, dropout_threshold,
                            keep_mask, mix32)


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _mix_scalar(x):
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7FEB352D) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846CA68B) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def _keep_scalar(seed, bh, n, i, j, T):
    rk = _mix_scalar((seed & 0xFFFFFFFF) ^ _mix_scalar((seed >> 32) ^ ((bh * n + i) & 0xFFFFFFFF)))
    w = _mix_scalar(rk ^ (((j >> 1) * 0x9E3779B9) & 0xFFFFFFFF))
    u = (w >> 16) & 0x7FFF if j & 1 else w & 0x7FFF
    return u >= T


def test_threshold_and_scale():
    assert dropout_threshold(0.0) == 0 and dropout_scale(0.0) == 1.0
    assert dropout_threshold(0.1) == 3277                      # 0.1 * 32768 = 3276.8
    assert abs(dropout_scale(0.1) - 1.0 / (1.0 - 3277 / 32768)) < 1e-15
    assert dropout_threshold(0.5) == 16384 and dropout_scale(0.5) == 2.0
    for bad in (-0.1, 1.0, 1.5, 0.99999):
        with pytest.raises(ValueError):
            dropout_threshold(bad)


def test_generator_integer_by_integer():
    seed, n = 0x1234_5678_9ABC_DEF0, 96
    for bh, p in ((0, 0.1), (5, 0.37), (1000, 0.9)):
        M = keep_mask(seed, bh, n, p)
        T = dropout_threshold(p)
        rng = np.random.default_rng(bh)
        for i, j in zip(rng.integers(0, n, 300), rng.integers(0, n, 300)):
            assert M[i, j] == _keep_scalar(seed, bh, n, int(i), int(j), T)
        rows = np.array([3, 95, 17])
        assert (keep_mask(seed, bh, n, p, rows=rows) == M[rows]).all()
    assert keep_mask(seed, 0, n, 0.0).all()
    # the row number wraps at 2^32 like the 32-bit arithmetic it stands for
    big_bh, n2 = 3_000_000, 2048
    M2 = keep_mask(7, big_bh, n2, 0.25, rows=[5])
    assert M2[0, 11] == _keep_scalar(7, big_bh, n2, 5, 11, dropout_threshold(0.25))


def test_mixing_function_has_no_collisions_and_avalanches():
    x = np.arange(1 << 20, dtype=np.uint32) + np.uint32(0xFFF00000)
    y = mix32(x)
    assert len(np.unique(y)) == len(x)
    flipped = mix32(x ^ np.uint32(1 << 7)) ^ y
    bits = np.unpackbits(flipped.view(np.uint8)).mean()
    assert abs(bits - 0.5) < 0.005


def test_keep_rate_and_independence():
    p, n = 0.1, 2048
    T = dropout_threshold(p)
    q = 1.0 - T / 32768.0
    M = keep_mask(99, 3, n, p)
    N = M.size
    sig = np.sqrt(q * (1 - q) / N)
    assert abs(M.mean() - q) < 4 * sig
    # per row and per column
    assert np.abs(M.mean(axis=1) - q).max() < 5.5 * np.sqrt(q * (1 - q) / n)
    assert np.abs(M.mean(axis=0) - q).max() < 5.5 * np.sqrt(q * (1 - q) / n)
    drop = ~M
    pd = 1 - q

    def joint_ok(a, b_):
        m = a.size
        both = (a & b_).mean()
        return abs(both - pd * pd) < 5 * np.sqrt(pd * pd * (1 - pd * pd) / m)

    assert joint_ok(drop[:, 0::2], drop[:, 1::2])          # the two numbers of one word
    assert joint_ok(drop[:, :-2], drop[:, 2:])             # neighbouring words
    assert joint_ok(drop[:-1, :], drop[1:, :])             # neighbouring rows
    assert joint_ok(drop, ~keep_mask(99, 4, n, p))         # neighbouring (batch, head) slices
    assert joint_ok(drop, ~keep_mask(100, 3, n, p))        # neighbouring seeds
    assert joint_ok(drop, ~keep_mask(99 + (1 << 32), 3, n, p))  # the seed's upper half counts


@pytest.mark.parametrize("mode", [oracle.GLOBAL_FIRST_LAST, oracle.GLOBAL_LEADING])
def test_p_zero_is_the_undropped_pass(mode):
    B, H, n, d, b, g, w, r = 2, 2, 48, 8, 4, 2, 3, 2
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 3, mode)
    Q, K, V, dO = (_rand((B, H, n, d), s) for s in (1, 2, 3, 4))
    km = np.ones((B, n), dtype=np.uint8)
    km[1, 29:] = 0
    O0, L0 = oracle.attn_fwd(Q, K, V, ridx, b, g, w, 0.4, key_mask=km, global_mode=mode)
    O1, L1 = attn_fwd_dropout(Q, K, V, ridx, b, g, w, 0.4, 0.0, 11, key_mask=km, global_mode=mode)
    assert (O0 == O1).all() and (L0 == L1).all()
    G0 = oracle.attn_bwd(Q, K, V, dO, ridx, b, g, w, 0.4, key_mask=km, global_mode=mode)
    G1 = attn_bwd_dropout(Q, K, V, dO, ridx, b, g, w, 0.4, 0.0, 11, key_mask=km, global_mode=mode)
    assert all((a == c).all() for a, c in zip(G0, G1))


def test_uniform_softmax_closed_form_by_loops():
    """Q = 0: every attended key has probability 1/|N(i)|; the output is the scaled mean of the
    kept value rows, taken here over the edge list with the scalar generator."""
    B, H, n, d, b, g, w, r = 1, 2, 40, 3, 4, 2, 3, 2
    p, seed = 0.3, 0xABCDEF0123
    T = dropout_threshold(p)
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 5)
    V = _rand((B, H, n, d), 9)
    K = _rand((B, H, n, d), 8)
    Q = np.zeros((B, H, n, d))
    km = np.ones((B, n), dtype=np.uint8)
    km[0, 33:] = 0
    O, LSE = attn_fwd_dropout(Q, K, V, ridx, b, g, w, 1.0, p, seed, key_mask=km)
    for h in range(H):
        for i in range(n):
            nbrs = [k * b + e for k in oracle.neighbour_blocks(ridx[h], n // b, i // b, g, w)
                    for e in range(b) if km[0, k * b + e]]
            acc = np.zeros(d)
            for j in nbrs:
                if _keep_scalar(seed, h, n, i, j, T):
                    acc += V[0, h, j]
            want = acc / len(nbrs) * (32768.0 / (32768.0 - T))
            assert np.abs(O[0, h, i] - want).max() < 1e-12
            assert abs(LSE[0, h, i] - np.log(len(nbrs))) < 1e-12


def test_mean_over_seeds_tends_to_the_undropped_output():
    B, H, n, d, b, g, w, r = 1, 1, 32, 4, 4, 2, 3, 1
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 2)
    Q, K, V = (_rand((B, H, n, d), s) for s in (5, 6, 7))
    O0, L0 = oracle.attn_fwd(Q, K, V, ridx, b, g, w, 0.5)
    n_seeds, p = 3000, 0.2
    acc = np.zeros_like(O0)
    sq = np.zeros_like(O0)
    for s in range(n_seeds):
        O, L = attn_fwd_dropout(Q, K, V, ridx, b, g, w, 0.5, p, s)
        assert (L == L0).all()
        acc += O
        sq += O * O
    mean = acc / n_seeds
    sem = np.sqrt(np.maximum(sq / n_seeds - mean * mean, 1e-30) / n_seeds)
    assert (np.abs(mean - O0) < 5.5 * sem + 1e-12).all()


def test_gradients_by_finite_differences_with_the_mask_fixed():
    B, H, n, d, b, g, w, r = 1, 2, 24, 4, 4, 2, 3, 1
    p, seed, scale = 0.25, 77, 0.6
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 4)
    Q, K, V, dO = (_rand((B, H, n, d), s) for s in (11, 12, 13, 14))
    km = np.ones((B, n), dtype=np.uint8)
    km[0, 21:] = 0
    dQ, dK, dV = attn_bwd_dropout(Q, K, V, dO, ridx, b, g, w, scale, p, seed, key_mask=km)

    def loss(q, k, v):
        return (attn_fwd_dropout(q, k, v, ridx, b, g, w, scale, p, seed, key_mask=km)[0] * dO).sum()

    rng = np.random.default_rng(0)
    eps = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(25):
            idx = tuple(rng.integers(0, s) for s in X.shape)
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - G[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, G[idx])
    # gradients of padded keys are exactly zero
    assert (dK[0, :, 21:] == 0).all() and (dV[0, :, 21:] == 0).all()


def test_sampled_rows_equal_the_full_evaluation():
    from oracle.dropout import attn_fwd_dropout_rows
    B, H, n, d, b, g, w, r = 2, 3, 48, 4, 4, 2, 3, 2
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 6)
    Q, K, V = (_rand((B, H, n, d), s) for s in (31, 32, 33))
    km = np.ones((B, n), dtype=np.uint8)
    km[1, 37:] = 0
    O, L = attn_fwd_dropout(Q, K, V, ridx, b, g, w, 0.3, 0.2, 99, key_mask=km)
    rows = [0, 5, 17, 46, 47]
    for bi, h in ((0, 0), (1, 2)):
        Or, Lr = attn_fwd_dropout_rows(Q, K, V, ridx, b, g, w, 0.3, 0.2, 99, bi, h, rows, key_mask=km)
        assert np.abs(Or - O[bi, h][rows]).max() < 1e-13 and np.abs(Lr - L[bi, h][rows]).max() < 1e-13


def test_row_sums_of_p_dp_equal_do_dot_o():
    B, H, n, d, b, g, w, r = 1, 1, 32, 5, 4, 2, 3, 1
    p, seed, scale = 0.4, 5, 0.7
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 1)
    Q, K, V, dO = (_rand((B, H, n, d), s) for s in (21, 22, 23, 24))
    O, _ = attn_fwd_dropout(Q, K, V, ridx, b, g, w, scale, p, seed)
    A = oracle.dense_mask(ridx[0], n, b, g, w)
    S = np.where(A, scale * Q[0, 0] @ K[0, 0].T, -np.inf)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    dP = np.where(keep_mask(seed, 0, n, p), dropout_scale(p), 0.0) * (dO[0, 0] @ V[0, 0].T)
    assert np.abs((P * dP).sum(axis=1) - (dO[0, 0] * O[0, 0]).sum(axis=1)).max() < 1e-12


def test_one_flipped_mask_bit_moves_the_counting_inputs_by_a_whole_step(monkeypatch):
    """The inputs of tests/test_dropout_mask_exact.py (uniform softmax, one-hot rows) make every
    output count kept pairs: a mistake planted here, one flipped bit of the oracle's mask, moves
    O, dV, dQ and dK by about one step each -- four times that test's tolerance."""
    import oracle.dropout as od
    B, H, n, b, g, w, r = 1, 2, 1024, 64, 2, 3, 3
    scale, p, seed = 0.125, 0.1, 0xC0FFEE1234
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 21)
    step = dropout_scale(p) / n
    oh = np.zeros((B, H, n, 64))
    oh[:, :, np.arange(n), np.arange(n) % 64] = 1.0
    z, ones = np.zeros((B, H, n, 64)), np.ones((B, H, n, 64))
    rnd = _rand((B, H, n, 64), 3)

    def run():
        return (od.attn_fwd_dropout(z, rnd, oh, ridx, b, g, w, scale, p, seed)[0],
                od.attn_bwd_dropout(z, rnd, oh, oh, ridx, b, g, w, scale, p, seed)[2],
                od.attn_bwd_dropout(z, oh, ones, ones / 64, ridx, b, g, w, scale, p, seed)[0],
                od.attn_bwd_dropout(oh, z, ones, ones / 64, ridx, b, g, w, scale, p, seed)[1])

    base = run()
    i, j = 5, 700                      # a global row (the smallest step) and some key
    orig = od.keep_mask

    def flipped(seed_, bh, n_, p_, rows=None):
        M = orig(seed_, bh, n_, p_, rows).copy()
        if bh == 1:
            rr = np.arange(n_) if rows is None else np.asarray(rows)
            k = np.flatnonzero(rr == i)
            if len(k):
                M[k[0], j] = ~M[k[0], j]
        return M

    monkeypatch.setattr(od, "keep_mask", flipped)
    new = run()
    for x, y, s in zip(new, base, (step, step, scale * step, scale * step)):
        assert np.abs(x - y).max() > 0.9 * s
