"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Every check here compares the oracle with something that is not the oracle:
per-element Python loops over an explicit edge list, closed forms, counts the
paper prints, finite differences.  A dropped term, wrong sign, transposed operand
or shifted index in oracle/ fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import (GLOBAL_FIRST_LAST, GLOBAL_LEADING, attn_bwd, attn_fwd, attn_fwd_rows,
                    count_block_pairs, dense_block_mask, dense_mask, global_blocks,
                    make_rand_idx, neighbour_blocks, reverse_random_lists, validate_rand_idx,
                    window_blocks)


# --------------------------------------------------------------------------- #
# helpers that share nothing with oracle/
# --------------------------------------------------------------------------- #
def read_paper_counts(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_pattern_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                vals[k] = int(v)
    return vals


def read_golden_table(golden_dir, name):
    with open(os.path.join(golden_dir, name + ".txt")) as f:
        H, nb, r, seed, g, w, mode = (int(x) for x in f.readline().split())
        rows = [[int(x) for x in line.split()] for line in f if line.strip()]
    return np.array(rows, dtype=np.int32).reshape(H, nb, r), (H, nb, r, seed, g, w, mode)


def loops_attention(q, k, v, edges, scale):
    """Eq. (AT) per head by per-element loops over an explicit list of (query, key) arcs."""
    n, d = len(q), len(q[0])
    out = [[0.0] * d for _ in range(n)]
    lse = [-math.inf] * n
    for i in range(n):
        nbrs = sorted(kk for (qq, kk) in edges if qq == i)
        if not nbrs:
            continue
        logits = [scale * sum(q[i][c] * k[j][c] for c in range(d)) for j in nbrs]
        mx = max(logits)
        ws = [math.exp(x - mx) for x in logits]
        tot = sum(ws)
        lse[i] = mx + math.log(tot)
        for wgt, j in zip(ws, nbrs):
            for c in range(d):
                out[i][c] += wgt / tot * v[j][c]
    return np.array(out), np.array(lse)


def figure_edge_list(n, b, g, w, rand_row_blocks, global_leading=True):
    """Arcs of the block pattern, enumerated token by token straight from App. D items 1-3."""
    nb = n // b
    half = (w - 1) // 2
    Gb = list(range(g)) if global_leading else None
    edges = set()
    for i in range(n):
        for k in range(n):
            jb, kb = i // b, k // b
            is_global = jb in Gb or kb in Gb
            is_window = abs(jb - kb) <= half
            is_random = kb in rand_row_blocks[jb]
            if is_global or is_window or is_random:
                edges.add((i, k))
    return edges


def rng_tensors(seed, *shape):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal(shape) for _ in range(3)]


# --------------------------------------------------------------------------- #
# pattern pins
# --------------------------------------------------------------------------- #
def test_keys_per_row_match_paper_counts(golden_dir):
    """App. D: (g+w+r)*b = 512 keys for an interior row of the ITC base pattern."""
    c = read_paper_counts(golden_dir)
    b, n = c["block_length_itc_base"], c["seq_len_itc_base"]
    nb = n // b
    tbl = make_rand_idx(2, n, b, 2, 3, c["random_blocks_all_experiments"], seed=1)
    for h in range(2):
        A = dense_mask(tbl[h], n, b, 2, 3)
        counts = A.sum(axis=1)
        assert (counts[2 * b:(nb - 2) * b] == c["keys_per_interior_row_itc_base"]).all()
        # blocks 1 and nb-2: the window holds a global block, counted once (A is 0/1)
        assert (counts[b:2 * b] == 7 * b).all() and (counts[(nb - 2) * b:(nb - 1) * b] == 7 * b).all()
        # global rows attend everything; global columns are attended by everyone (Sec. 2, ITC)
        assert (counts[:b] == n).all() and (counts[(nb - 1) * b:] == n).all()
        assert A[:, :b].all() and A[:, (nb - 1) * b:].all()
        assert int(A.sum()) == b * b * (10 * nb - 18)
    assert count_block_pairs(tbl, n, b, 2, 3) == 2 * (10 * nb - 18)


def test_figure_example_sizes(golden_dir):
    """App. D worked example: 12 tokens, block 2 -> 6x6 blocks; r=1, w=3, g=1."""
    c = read_paper_counts(golden_dir)
    n, b = c["figure_tokens"], 2
    nb = n // b
    assert nb == c["figure_blocks"]
    tbl = make_rand_idx(1, n, b, 1, 3, 1, seed=7)
    Mb = dense_block_mask(tbl[0], nb, 1, 3)
    assert Mb.shape == (6, 6)
    assert Mb[0].all() and Mb[:, 0].all()
    for j in range(2, nb - 1):
        assert Mb[j].sum() == c["figure_interior_row_blocks"]
        assert Mb[j, j - 1] and Mb[j, j] and Mb[j, j + 1]


def test_window_definition():
    assert window_blocks(10, 4, 3) == [3, 4, 5]
    assert window_blocks(10, 0, 3) == [0, 1]
    assert window_blocks(10, 9, 5) == [7, 8, 9]
    with pytest.raises(ValueError):
        window_blocks(10, 4, 2)


def test_global_placements():
    assert global_blocks(8, 2, GLOBAL_FIRST_LAST) == [0, 7]
    assert global_blocks(8, 1, GLOBAL_FIRST_LAST) == [0]
    assert global_blocks(8, 3, GLOBAL_FIRST_LAST) == [0, 1, 7]
    assert global_blocks(8, 3, GLOBAL_LEADING) == [0, 1, 2]
    assert global_blocks(8, 0, GLOBAL_FIRST_LAST) == []


def test_clipped_and_circular_window_agree_when_ends_are_global():
    """App. D builds the window by a circular roll; with first and last block global the
    wrapped blocks are global anyway, so the clipped band gives the same sets (w <= 5 needs g >= 4)."""
    nb, g, w = 16, 2, 3
    G = set(global_blocks(nb, g))
    half = (w - 1) // 2
    for j in range(nb):
        circ = {(j + o) % nb for o in range(-half, half + 1)} | G
        clip = set(window_blocks(nb, j, w)) | G
        assert circ == clip


def test_rand_idx_properties_and_determinism():
    H, n, b, g, w, r = 3, 2048, 64, 2, 3, 3
    nb = n // b
    t = make_rand_idx(H, n, b, g, w, r, seed=5)
    assert t.dtype == np.int32 and t.shape == (H, nb, r)
    assert validate_rand_idx(t, H, n, b, g, w, r)
    G = set(global_blocks(nb, g))
    for h in range(H):
        for j in range(nb):
            row = list(t[h, j])
            if j in G:
                assert row == [-1] * r
                continue
            assert row == sorted(row) and len(set(row)) == r          # "exactly r random blocks"
            assert all(0 <= k < nb for k in row)
            assert not (set(row) & (G | {j - 1, j, j + 1}))
    assert (make_rand_idx(H, n, b, g, w, r, seed=5) == t).all()
    assert (make_rand_idx(H, n, b, g, w, r, seed=6) != t).any()
    assert (t[0] != t[1]).any()
    bad = t.copy()
    bad[0, 5, 0] = 5
    assert not validate_rand_idx(bad, H, n, b, g, w, r)
    bad = t.copy()
    bad[1, 7, 1] = bad[1, 7, 0]
    assert not validate_rand_idx(bad, H, n, b, g, w, r)
    with pytest.raises(ValueError):
        make_rand_idx(1, 5 * 64, 64, 2, 3, 3, seed=0)     # block 2 has no candidate left


def test_rand_idx_leading_globals_properties():
    """The App. D wording ("the first g blocks are global"): same rules, other global set, checked by
    an inline loop that uses nothing from the oracle but the table."""
    H, n, b, g, w, r = 2, 1536, 64, 3, 5, 2
    nb = n // b
    t = make_rand_idx(H, n, b, g, w, r, seed=8, global_mode=GLOBAL_LEADING)
    assert t.dtype == np.int32 and t.shape == (H, nb, r)
    picked = np.zeros(nb, dtype=np.int64)
    for h in range(H):
        for j in range(nb):
            row = [int(x) for x in t[h, j]]
            if j < g:                                  # blocks 0 .. g-1 are the global ones
                assert row == [-1] * r
                continue
            assert row == sorted(row) and len(set(row)) == r
            for k in row:
                assert g <= k < nb                     # never a global block
                assert abs(k - j) > (w - 1) // 2       # never inside the window
                picked[k] += 1
    assert picked[nb - 1] > 0                          # the last block is an ordinary one here
    assert (make_rand_idx(H, n, b, g, w, r, seed=8, global_mode=GLOBAL_LEADING) == t).all()
    assert (make_rand_idx(H, n, b, g, w, r, seed=8, global_mode=GLOBAL_FIRST_LAST) != t).any()
    assert validate_rand_idx(t, H, n, b, g, w, r, GLOBAL_LEADING)
    assert not validate_rand_idx(t, H, n, b, g, w, r, GLOBAL_FIRST_LAST)   # nb-1 is global there


def test_count_block_pairs_by_double_loop_and_closed_forms():
    """count_block_pairs, with and without a key-block validity vector, against (i) a double loop over
    (j, k) written from the three set definitions (Sec. 2 globals, App. D window and random
    blocks), (ii) the closed form P(nb) = 10 nb - 18 for g/w/r = 2/3/3 and (iii), for a valid prefix
    of L blocks, the count derived by hand below."""
    H, n, b, g, w, r = 3, 2048, 64, 2, 3, 3
    nb = n // b
    t = make_rand_idx(H, n, b, g, w, r, seed=12)

    def loop_count(valid):
        total = 0
        for h in range(H):
            for j in range(nb):
                for k in range(nb):
                    is_g_row = j == 0 or j == nb - 1
                    is_g_col = k == 0 or k == nb - 1
                    in_win = abs(k - j) <= 1
                    in_rnd = any(int(x) == k for x in t[h, j])
                    if (is_g_row or is_g_col or in_win or in_rnd) and valid[k]:
                        total += 1
        return total

    all_valid = np.ones(nb, dtype=bool)
    assert count_block_pairs(t, n, b, g, w) == loop_count(all_valid) == H * (10 * nb - 18)
    rng = np.random.default_rng(3)
    for _ in range(4):
        valid = rng.random(nb) < 0.6
        assert count_block_pairs(t, n, b, g, w, key_block_valid=valid) == loop_count(valid)
    # Valid prefix of L blocks, 2 <= L <= nb - 2 (the last global block is padded).  Per head:
    #   the two global rows see L valid blocks each;
    #   every other row sees block 0;
    #   window: rows 1 .. L-1 see themselves (L-1 pairs), rows 2 .. L see j-1 with j-1 >= 1
    #   (L-1 pairs), rows 1 .. L-2 see j+1 <= L-1 (L-2 pairs); block 0 as a window block of row 1
    #   is the global pair already counted;
    #   random: counted from the table (entries < L), they never coincide with the above.
    for L in (2, 5, 17, nb - 2):
        valid = np.arange(nb) < L
        rand_pairs = sum(int(0 <= int(x) < L) for h in range(H) for j in range(1, nb - 1) for x in t[h, j])
        by_hand = H * (2 * L + (nb - 2) + (L - 1) + (L - 1) + (L - 2)) + rand_pairs
        assert count_block_pairs(t, n, b, g, w, key_block_valid=valid) == by_hand
        assert loop_count(valid) == by_hand


def test_rand_idx_uniform_over_candidates():
    """Chi-square of picks over the candidate blocks of one row, across many heads."""
    H, n, b, g, w, r = 4000, 16 * 64, 64, 2, 3, 3
    t = make_rand_idx(H, n, b, g, w, r, seed=11)
    j = 8
    cand = [k for k in range(16) if k not in (0, 15, 7, 8, 9)]
    counts = np.array([(t[:, j, :] == k).sum() for k in cand], dtype=np.float64)
    assert counts.sum() == H * r
    expect = H * r / len(cand)
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 35.0          # 10 degrees of freedom: P(chi2 > 35) ~ 1e-4
    # pairs are uniform too (without replacement): no pair of equal picks
    assert all(len(set(row)) == r for row in t[:, j, :])


def test_rand_idx_matches_golden_files(golden_dir):
    for name in ["rand_idx_cfg1_seed0", "rand_idx_cfg2_seed1", "rand_idx_cfg5_seed4_head0_3",
                 "rand_idx_figure_seed7", "rand_idx_leading_seed9"]:
        want, (H, nb, r, seed, g, w, mode) = read_golden_table(golden_dir, name)
        b = 2 if "figure" in name else 64
        got = make_rand_idx(H, nb * b, b, g, w, r, seed, mode)
        assert (got == want).all(), name


def test_reverse_lists_are_the_inverse_relation():
    H, n, b, g, w, r = 2, 4096, 64, 2, 3, 3
    nb = n // b
    t = make_rand_idx(H, n, b, g, w, r, seed=3)
    for h in range(H):
        rev = reverse_random_lists(t[h], nb)
        fwd_pairs = sorted((j, int(k)) for j in range(nb) for k in t[h, j] if k >= 0)
        rev_pairs = sorted((j, k) for k in range(nb) for j in rev[k])
        assert fwd_pairs == rev_pairs
        assert sum(len(x) for x in rev) == (nb - g) * r
        assert all(x == sorted(x) for x in rev)


# --------------------------------------------------------------------------- #
# forward pins
# --------------------------------------------------------------------------- #
def test_brute_force_at_figure_size():
    """n=12, b=2, g=1 (leading), w=3, r=1: per-element loops over the explicit arc list."""
    n, b, g, w, r, d = 12, 2, 1, 3, 1, 3
    tbl = make_rand_idx(1, n, b, g, w, r, seed=7, global_mode=GLOBAL_LEADING)
    rand_rows = [[int(k) for k in tbl[0, j] if k >= 0] for j in range(n // b)]
    edges = figure_edge_list(n, b, g, w, rand_rows)
    Q, K, V = rng_tensors(0, 1, 1, n, d)
    scale = 0.7
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, scale, global_mode=GLOBAL_LEADING)
    Oref, Lref = loops_attention(Q[0, 0].tolist(), K[0, 0].tolist(), V[0, 0].tolist(), edges, scale)
    np.testing.assert_allclose(O[0, 0], Oref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE[0, 0], Lref, rtol=0, atol=1e-12)


def test_brute_force_two_heads_first_last_and_padding():
    n, b, g, w, r, d = 32, 4, 2, 3, 2, 5
    nb = n // b
    tbl = make_rand_idx(2, n, b, g, w, r, seed=13)
    Q, K, V = rng_tensors(1, 2, 2, n, d)
    key_mask = np.ones((2, n), dtype=np.uint8)
    key_mask[1, 22:] = 0
    scale = 1.0 / math.sqrt(d)
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, scale, key_mask=key_mask)
    for bi in range(2):
        for h in range(2):
            edges = set()
            for i in range(n):
                for k in range(n):
                    jb, kb = i // b, k // b
                    if (jb in (0, nb - 1) or kb in (0, nb - 1) or abs(jb - kb) <= 1
                            or kb in tbl[h, jb]) and key_mask[bi, k]:
                        edges.add((i, k))
            Oref, Lref = loops_attention(Q[bi, h].tolist(), K[bi, h].tolist(), V[bi, h].tolist(),
                                         edges, scale)
            np.testing.assert_allclose(O[bi, h], Oref, rtol=0, atol=1e-12)
            np.testing.assert_allclose(LSE[bi, h], Lref, rtol=0, atol=1e-12)


def test_full_coverage_equals_textbook_attention():
    """Sec. 2: A all ones recovers full attention.  Widen the window to cover every block."""
    n, b, d = 24, 4, 6
    nb = n // b
    Q, K, V = rng_tensors(2, 1, 2, n, d)
    scale = 0.4
    all_edges = {(i, k) for i in range(n) for k in range(n)}
    empty = np.full((2, nb, 0), -1, dtype=np.int32)
    for (g, w) in [(0, 2 * nb - 1), (nb, 1), (2, 2 * nb + 1)]:
        O, LSE = attn_fwd(Q, K, V, empty, b, g, w, scale)
        for h in range(2):
            Oref, Lref = loops_attention(Q[0, h].tolist(), K[0, h].tolist(), V[0, h].tolist(),
                                         all_edges, scale)
            np.testing.assert_allclose(O[0, h], Oref, rtol=0, atol=1e-12)
            np.testing.assert_allclose(LSE[0, h], Lref, rtol=0, atol=1e-12)


def test_zero_queries_closed_form_and_pattern_readback():
    """Q = 0: uniform weights over N(i), O_i = mean of V over N(i), LSE_i = ln |N(i)|.
    With V[k, c] = [k // b == c] the output spells out the neighbour set of every row."""
    H, n, b, g, w, r = 2, 1024, 64, 2, 3, 3
    nb = n // b
    d = nb
    tbl = make_rand_idx(H, n, b, g, w, r, seed=0)
    Q = np.zeros((1, H, n, d))
    K = np.random.default_rng(3).standard_normal((1, H, n, d))
    V = np.zeros((1, H, n, d))
    for k in range(n):
        V[:, :, k, k // b] = 1.0
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, 0.125)
    for h in range(H):
        for j in range(nb):
            if j in (0, nb - 1):
                want = set(range(nb))
            else:
                want = {0, nb - 1, j - 1, j, j + 1} | {int(x) for x in tbl[h, j]}
            cnt = len(want) * b
            row = O[0, h, j * b + 5]
            assert {c for c in range(d) if row[c] > 0} == want
            np.testing.assert_allclose(row[sorted(want)], b / cnt, rtol=1e-13)
            np.testing.assert_allclose(LSE[0, h, j * b:(j + 1) * b], math.log(cnt), rtol=1e-13)
    assert math.isclose(LSE[0, 0, 3 * b], math.log(512)) and math.isclose(LSE[0, 0, b], math.log(448))


def test_softmax_normalisation_and_shift_properties():
    H, n, b, g, w, r, d = 2, 256, 16, 2, 3, 3, 8
    tbl = make_rand_idx(H, n, b, g, w, r, seed=2)
    Q, K, V = rng_tensors(4, 2, H, n, d)
    scale = 0.3
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, scale)
    # sum_k exp(S_ik - LSE_i) = 1 over N(i), recomputed here without the oracle's softmax
    for (bi, h, i) in [(0, 0, 0), (1, 1, 17), (0, 1, 100), (1, 0, 255), (0, 0, 31)]:
        nbr = neighbour_blocks(tbl[h], n // b, i // b, g, w)
        keys = [k for kb in nbr for k in range(kb * b, (kb + 1) * b)]
        s = sum(math.exp(scale * float(Q[bi, h, i] @ K[bi, h, k]) - LSE[bi, h, i]) for k in keys)
        assert abs(s - 1.0) < 1e-12
    # V -> V + c shifts O by c
    O2, LSE2 = attn_fwd(Q, K, V + 2.5, tbl, b, g, w, scale)
    np.testing.assert_allclose(O2, O + 2.5, atol=1e-12)
    np.testing.assert_allclose(LSE2, LSE, atol=1e-12)
    # adding a constant vector u to every key adds scale*q.u to all logits of a row:
    # O unchanged, LSE shifted by exactly that amount
    u = np.random.default_rng(5).standard_normal(d)
    O3, LSE3 = attn_fwd(Q, K + u, V, tbl, b, g, w, scale)
    np.testing.assert_allclose(O3, O, atol=1e-11)
    np.testing.assert_allclose(LSE3, LSE + scale * (Q @ u), atol=1e-11)


def test_random_row_order_does_not_matter():
    H, n, b, g, w, r, d = 1, 512, 32, 2, 3, 3, 4
    tbl = make_rand_idx(H, n, b, g, w, r, seed=8)
    Q, K, V = rng_tensors(6, 1, H, n, d)
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, 0.5)
    O2, LSE2 = attn_fwd(Q, K, V, tbl[:, :, ::-1].copy(), b, g, w, 0.5)
    np.testing.assert_allclose(O2, O, atol=1e-13)


def test_padding_equals_truncated_key_set():
    """Masking keys [L, n) equals attention over keys [0, L) with each N(i) cut to [0, L)."""
    H, n, b, g, w, r, d = 1, 256, 16, 2, 3, 3, 8
    nb = n // b
    tbl = make_rand_idx(H, n, b, g, w, r, seed=9)
    Q, K, V = rng_tensors(7, 1, H, n, d)
    L = 9 * b + 5                                  # not block aligned on purpose
    km = np.zeros((1, n), dtype=np.uint8)
    km[0, :L] = 1
    scale = 0.35
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, scale, key_mask=km)
    edges = set()
    for i in range(n):
        for kb in neighbour_blocks(tbl[0], nb, i // b, g, w):
            for k in range(kb * b, (kb + 1) * b):
                if k < L:
                    edges.add((i, k))
    Oref, Lref = loops_attention(Q[0, 0].tolist(), K[0, 0].tolist(), V[0, 0].tolist(), edges, scale)
    np.testing.assert_allclose(O[0, 0], Oref, atol=1e-12)
    np.testing.assert_allclose(LSE[0, 0], Lref, atol=1e-12)


def test_row_without_valid_keys():
    H, n, b, g, w, r, d = 1, 64, 8, 1, 1, 0, 4
    tbl = np.full((H, n // b, 0), -1, dtype=np.int32)
    Q, K, V = rng_tensors(8, 1, H, n, d)
    km = np.ones((1, n), dtype=np.uint8)
    km[0, :8] = 0            # global block 0 padded
    km[0, 24:32] = 0         # block 3 padded: its own rows see nothing (g=1 -> only block 0 and self)
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, 1.0, key_mask=km, global_mode=GLOBAL_LEADING)
    assert (O[0, 0, 24:32] == 0).all() and np.isneginf(LSE[0, 0, 24:32]).all()
    assert np.isfinite(LSE[0, 0, 32:40]).all()
    dQ, dK, dV = attn_bwd(Q, K, V, np.ones_like(Q), tbl, b, g, w, 1.0, key_mask=km,
                          global_mode=GLOBAL_LEADING)
    assert (dQ[0, 0, 24:32] == 0).all()
    assert (dK[0, 0, :8] == 0).all() and (dV[0, 0, :8] == 0).all()
    assert (dK[0, 0, 24:32] == 0).all() and (dV[0, 0, 24:32] == 0).all()


def test_rows_subset_matches_full():
    H, n, b, g, w, r, d = 2, 512, 32, 2, 3, 3, 8
    tbl = make_rand_idx(H, n, b, g, w, r, seed=10)
    Q, K, V = rng_tensors(9, 2, H, n, d)
    km = np.ones((2, n), dtype=np.uint8)
    km[1, 400:] = 0
    O, LSE = attn_fwd(Q, K, V, tbl, b, g, w, 0.25, key_mask=km)
    rows = [0, 31, 32, 77, 300, 511]
    Or, Lr = attn_fwd_rows(Q, K, V, tbl, b, g, w, 0.25, 1, 1, rows, key_mask=km)
    np.testing.assert_allclose(Or, O[1, 1, rows], atol=1e-13)
    np.testing.assert_allclose(Lr, LSE[1, 1, rows], atol=1e-13)


# --------------------------------------------------------------------------- #
# backward pins (the paper gives no backward pass: calculus on eq. (AT))
# --------------------------------------------------------------------------- #
def _loss_via_loops(Q, K, V, dO, edges, scale):
    O, _ = loops_attention(Q.tolist(), K.tolist(), V.tolist(), edges, scale)
    return float((O * dO).sum())


def test_gradients_match_central_differences_of_independent_forward():
    n, b, g, w, r, d = 16, 2, 2, 3, 1, 3
    nb = n // b
    tbl = make_rand_idx(1, n, b, g, w, r, seed=21)
    rng = np.random.default_rng(10)
    Q, K, V, dO = (rng.standard_normal((1, 1, n, d)) for _ in range(4))
    km = np.ones((1, n), dtype=np.uint8)
    km[0, 11] = 0
    scale = 0.6
    dQ, dK, dV = attn_bwd(Q, K, V, dO, tbl, b, g, w, scale, key_mask=km)
    edges = {(i, k) for i in range(n) for k in range(n)
             if km[0, k] and (k // b) in neighbour_blocks(tbl[0], nb, i // b, g, w)}
    eps = 1e-6
    probes = [(0, 0), (3, 1), (7, 2), (11, 0), (15, 1), (8, 2)]
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for (i, c) in probes:
            args = {"Q": Q[0, 0].copy(), "K": K[0, 0].copy(), "V": V[0, 0].copy()}
            args[name][i, c] += eps
            up = _loss_via_loops(args["Q"], args["K"], args["V"], dO[0, 0], edges, scale)
            args[name][i, c] -= 2 * eps
            dn = _loss_via_loops(args["Q"], args["K"], args["V"], dO[0, 0], edges, scale)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - G[0, 0, i, c]) <= 1e-6 * max(1.0, abs(fd)), (name, i, c, fd, G[0, 0, i, c])
    assert (dK[0, 0, 11] == 0).all() and (dV[0, 0, 11] == 0).all()


def test_zero_queries_dV_closed_form():
    """Q = 0: P is uniform on N(i), so dV_k = sum over rows i with k in N(i) of dO_i / |N(i)|,
    and dK = scale * dS^T Q = 0."""
    H, n, b, g, w, r, d = 1, 128, 8, 2, 3, 2, 4
    nb = n // b
    tbl = make_rand_idx(H, n, b, g, w, r, seed=4)
    rng = np.random.default_rng(11)
    K, V, dO = (rng.standard_normal((1, H, n, d)) for _ in range(3))
    Q = np.zeros_like(K)
    dQ, dK, dV = attn_bwd(Q, K, V, dO, tbl, b, g, w, 0.5)
    want = np.zeros((n, d))
    for i in range(n):
        nbr = neighbour_blocks(tbl[0], nb, i // b, g, w)
        for kb in nbr:
            want[kb * b:(kb + 1) * b] += dO[0, 0, i] / (len(nbr) * b)
    np.testing.assert_allclose(dV[0, 0], want, atol=1e-13)
    assert np.abs(dK).max() == 0.0


def test_gradient_invariances():
    """Logit shift invariance: the loss does not change when a constant vector is added to all
    keys, so sum_k dK_k = 0; and sum over keys of dV equals sum over queries of dO (rows of P sum to 1)."""
    H, n, b, g, w, r, d = 2, 256, 16, 2, 3, 3, 8
    tbl = make_rand_idx(H, n, b, g, w, r, seed=12)
    rng = np.random.default_rng(12)
    Q, K, V, dO = (rng.standard_normal((1, H, n, d)) for _ in range(4))
    dQ, dK, dV = attn_bwd(Q, K, V, dO, tbl, b, g, w, 0.3)
    # sum_k dK_k = scale * sum_i (sum_k dS_ik) q_i and each row of dS sums to zero
    np.testing.assert_allclose(dK.sum(axis=2), 0.0, atol=1e-11)
    np.testing.assert_allclose(dV.sum(axis=2), dO.sum(axis=2), atol=1e-11)


def test_backward_full_coverage_matches_dense_formula_by_loops():
    """With every block attended the gradients are those of textbook attention; checked
    against per-element sums written from the softmax Jacobian."""
    n, b, d = 8, 2, 2
    nb = n // b
    rng = np.random.default_rng(13)
    Q, K, V, dO = (rng.standard_normal((1, 1, n, d)) for _ in range(4))
    scale = 0.9
    empty = np.full((1, nb, 0), -1, dtype=np.int32)
    dQ, dK, dV = attn_bwd(Q, K, V, dO, empty, b, 0, 2 * nb - 1, scale)
    q, k, v, do = Q[0, 0], K[0, 0], V[0, 0], dO[0, 0]
    P = np.zeros((n, n))
    for i in range(n):
        e = [math.exp(scale * float(q[i] @ k[j])) for j in range(n)]
        P[i] = np.array(e) / sum(e)
    wantQ, wantK, wantV = np.zeros((n, d)), np.zeros((n, d)), np.zeros((n, d))
    for i in range(n):
        for j in range(n):
            wantV[j] += P[i, j] * do[i]
            dp_ij = float(do[i] @ v[j])
            Di = sum(P[i, t] * float(do[i] @ v[t]) for t in range(n))
            ds = P[i, j] * (dp_ij - Di)
            wantQ[i] += scale * ds * k[j]
            wantK[j] += scale * ds * q[i]
    np.testing.assert_allclose(dQ[0, 0], wantQ, atol=1e-12)
    np.testing.assert_allclose(dK[0, 0], wantK, atol=1e-12)
    np.testing.assert_allclose(dV[0, 0], wantV, atol=1e-12)


def test_scale_invariance_identity_of_the_gradients():
    """S depends on Q and K only through Q K^T, so sum(Q o dQ) = sum(K o dK) per head (both equal
    sum(dS o S)).  A wrong transpose, a dropped scale or a missing -D term breaks it."""
    H, n, b, g, w, r, d = 2, 256, 16, 1, 3, 2, 8
    tbl = make_rand_idx(H, n, b, g, w, r, seed=5)
    rng = np.random.default_rng(5)
    Q, K, V, dO = (rng.standard_normal((1, H, n, d)) for _ in range(4))
    dQ, dK, dV = attn_bwd(Q, K, V, dO, tbl, b, g, w, 0.3)
    qdq = (Q * dQ).sum(axis=(2, 3))
    kdk = (K * dK).sum(axis=(2, 3))
    np.testing.assert_allclose(qdq, kdk, rtol=1e-10, atol=1e-10)
    assert np.abs(qdq).min() > 1e-3  # not trivially zero
