"""Pins of the oracle's skip_padded_query_blocks option -- CPU only.

The option reads the key-padding mask also as a query mask, block by block: a query block in
which every position is padded has no neighbours (O = 0, LSE = -inf, no gradient through it);
every other row is untouched.  Pinned by things other than the option's own code:
  * rows of blocks with a valid position are bit-identical to the run without the option, rows
    of fully padded blocks are exactly 0 / -inf (per-element comparison written out here);
  * for a padded suffix that ends on a block boundary, the valid rows equal plain attention on
    the truncated sequence with the pattern's key sets cut to it (an independent loop);
  * gradients: the option equals the plain backward fed with dO = 0 on the skipped rows, and
    central finite differences of the forward with the option;
  * the pair count drops by exactly the pairs of the skipped query blocks (counted by loops).
"""
import numpy as np
import pytest

import oracle


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _setup(B=2, H=2, n=48, d=5, b=4, g=2, w=3, r=2, seed=3, mode=oracle.GLOBAL_FIRST_LAST):
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, seed, mode)
    Q, K, V, dO = (_rand((B, H, n, d), s) for s in (1, 2, 3, 4))
    km = np.ones((B, n), dtype=np.uint8)
    km[0, 30:] = 0          # blocks 8.. of 12 fully padded, block 7 half padded
    km[1, 4:9] = 0          # a hole: block 1 (rows 4..7) fully padded, row 8 of block 2 as well
    km[1, 44:] = 0          # last (global) block fully padded
    return ridx, Q, K, V, dO, km, (b, g, w)


@pytest.mark.parametrize("mode", [oracle.GLOBAL_FIRST_LAST, oracle.GLOBAL_LEADING])
def test_only_rows_of_fully_padded_blocks_change(mode):
    ridx, Q, K, V, dO, km, (b, g, w) = _setup(mode=mode)
    O0, L0 = oracle.attn_fwd(Q, K, V, ridx, b, g, w, 0.4, key_mask=km, global_mode=mode)
    O1, L1 = oracle.attn_fwd(Q, K, V, ridx, b, g, w, 0.4, key_mask=km, global_mode=mode,
                             skip_padded_query_blocks=True)
    B, H, n, _ = Q.shape
    n_skipped = 0
    for bi in range(B):
        for i in range(n):
            j = i // b
            padded_block = not any(km[bi, j * b + e] for e in range(b))
            for h in range(H):
                if padded_block:
                    n_skipped += 1
                    assert (O1[bi, h, i] == 0).all() and L1[bi, h, i] == -np.inf
                else:
                    assert (O1[bi, h, i] == O0[bi, h, i]).all() and L1[bi, h, i] == L0[bi, h, i]
    assert n_skipped == H * (16 + 4 + 4)   # batch 0: blocks 8..11; batch 1: blocks 1 and 11
    rows = [0, 5, 29, 31, 32, 47]
    for bi, h in ((0, 1), (1, 0)):
        Or, Lr = oracle.attn_fwd_rows(Q, K, V, ridx, b, g, w, 0.4, bi, h, rows, key_mask=km,
                                      global_mode=mode, skip_padded_query_blocks=True)
        assert (Or == O1[bi, h][rows]).all() or np.abs(Or - O1[bi, h][rows]).max() < 1e-13
        assert (Lr == L1[bi, h][rows]).all() or np.abs(Lr[np.isfinite(Lr)] - L1[bi, h][rows][np.isfinite(Lr)]).max() < 1e-13


def test_aligned_suffix_equals_attention_on_the_truncated_sequence():
    """Valid length 32 of 48 (8 of 12 blocks): a valid row attends its pattern's blocks below 8."""
    b, g, w, r, H, n, d, Lv = 4, 2, 3, 2, 2, 48, 3, 32
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 9)
    Q, K, V = (_rand((1, H, n, d), s) for s in (5, 6, 7))
    km = np.zeros((1, n), dtype=np.uint8)
    km[0, :Lv] = 1
    O, L = oracle.attn_fwd(Q, K, V, ridx, b, g, w, 0.7, key_mask=km, skip_padded_query_blocks=True)
    for h in range(H):
        for i in range(n):
            if i >= Lv:
                assert (O[0, h, i] == 0).all() and L[0, h, i] == -np.inf
                continue
            keys = [k * b + e for k in oracle.neighbour_blocks(ridx[h], n // b, i // b, g, w)
                    for e in range(b) if k * b + e < Lv]
            s = np.array([0.7 * float(Q[0, h, i] @ K[0, h, j]) for j in keys])
            pr = np.exp(s - s.max())
            pr /= pr.sum()
            want = sum(pj * V[0, h, j] for pj, j in zip(pr, keys))
            assert np.abs(O[0, h, i] - want).max() < 1e-12
            assert abs(L[0, h, i] - (s.max() + np.log(np.exp(s - s.max()).sum()))) < 1e-12


def test_gradients_are_those_of_the_plain_pass_with_zero_upstream_on_skipped_rows():
    ridx, Q, K, V, dO, km, (b, g, w) = _setup()
    G1 = oracle.attn_bwd(Q, K, V, dO, ridx, b, g, w, 0.4, key_mask=km, skip_padded_query_blocks=True)
    B, H, n, _ = Q.shape
    dO0 = dO.copy()
    skipped = np.zeros((B, n), dtype=bool)
    for bi in range(B):
        for j in range(n // b):
            if not km[bi, j * b:(j + 1) * b].any():
                skipped[bi, j * b:(j + 1) * b] = True
    dO0[np.broadcast_to(skipped[:, None, :], (B, H, n))] = 0.0
    G0 = oracle.attn_bwd(Q, K, V, dO0, ridx, b, g, w, 0.4, key_mask=km)
    # dK, dV: the skipped rows send nothing either way; dQ: their own rows are zero with the option,
    # and zero in the plain pass too once their upstream gradient is zero
    for a, c in zip(G1, G0):
        assert np.abs(a - c).max() < 1e-13
    assert (G1[0][np.broadcast_to(skipped[:, None, :], (B, H, n))] == 0).all()

    def loss(q, k, v):
        return (oracle.attn_fwd(q, k, v, ridx, b, g, w, 0.4, key_mask=km, skip_padded_query_blocks=True)[0] * dO).sum()

    rng = np.random.default_rng(1)
    eps = 1e-6
    for name, X, G in (("Q", Q, G1[0]), ("K", K, G1[1]), ("V", V, G1[2])):
        for _ in range(20):
            idx = tuple(rng.integers(0, s) for s in X.shape)
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            ap = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            am = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*ap) - loss(*am)) / (2 * eps)
            assert abs(fd - G[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx)


def test_pair_count_drops_by_the_pairs_of_the_skipped_query_blocks():
    b, g, w, r, H, n = 4, 2, 3, 2, 3, 64
    nb = n // b
    ridx = oracle.make_rand_idx(H, n, b, g, w, r, 4)
    valid = np.ones(nb, dtype=bool)
    valid[10:] = False
    valid[3] = False
    full = oracle.count_block_pairs(ridx, n, b, g, w, key_block_valid=valid)
    skip = oracle.count_block_pairs(ridx, n, b, g, w, key_block_valid=valid, skip_padded_query_blocks=True)
    dropped = 0
    for h in range(H):
        for j in range(nb):
            if not valid[j]:
                dropped += sum(1 for k in oracle.neighbour_blocks(ridx[h], nb, j, g, w) if valid[k])
    assert full - skip == dropped and dropped > 0
