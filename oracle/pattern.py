"""The BigBird block pattern, written out from its definition.  TEST INFRASTRUCTURE ONLY.

Sec. 2 defines the graph as the union of three components -- random keys, a
sliding window and global tokens (ITC: a subset G of existing tokens with full
rows and full columns of the adjacency matrix A).  App. D restates all three on
blocks of b tokens: query block j attends r random key blocks, key blocks
j-(w-1)/2 .. j+(w-1)/2, and the g global blocks; global query blocks attend
every key block.

Readings taken where the paper is silent (listed in the design notes):
  * which blocks are global: "first and last" placement puts ceil(g/2) blocks at
    the start and floor(g/2) at the end; "leading" uses the first g (App. D text);
  * the window is clipped at the sequence ends (Sec. 2 band), not wrapped;
  * components overlap as a set union: A is 0/1, each key is counted once;
  * random blocks of a query block are drawn uniformly without replacement from
    the key blocks outside its window and outside G; one table per head.
"""
from __future__ import annotations

import numpy as np

GLOBAL_FIRST_LAST = 0
GLOBAL_LEADING = 1

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_HEAD_MUL = 0xD6E8FEB86659FD93
_ROW_MUL = 0xA0761D6478BD642F


# --------------------------------------------------------------------------- #
# Block sets (App. D, items 1-3)
# --------------------------------------------------------------------------- #
def global_blocks(nb: int, g: int, global_mode: int = GLOBAL_FIRST_LAST) -> list[int]:
    """Indices of the g global blocks (ITC: existing tokens made global, Sec. 2)."""
    if g < 0 or g > nb:
        raise ValueError("need 0 <= g <= nb")
    if global_mode == GLOBAL_LEADING:
        return list(range(g))
    if global_mode == GLOBAL_FIRST_LAST:
        lead = (g + 1) // 2
        trail = g // 2
        return list(range(lead)) + list(range(nb - trail, nb))
    raise ValueError("unknown global_mode")


def window_blocks(nb: int, j: int, w: int) -> list[int]:
    """Key blocks j-(w-1)/2 .. j+(w-1)/2 including j, clipped to [0, nb) (App. D item 2)."""
    if w < 1 or w % 2 == 0:
        raise ValueError("w must be odd and >= 1")
    half = (w - 1) // 2
    return [k for k in range(j - half, j + half + 1) if 0 <= k < nb]


# --------------------------------------------------------------------------- #
# Random-block table: a counter-based integer generator, no floating point
# --------------------------------------------------------------------------- #
def _mix64(z: int) -> int:
    """64-bit finaliser of the SplitMix64 generator (Steele, Lea, Flood 2014)."""
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _row_key(seed: int, h: int, j: int) -> int:
    k = _mix64(seed + _GOLDEN)
    k = _mix64(k ^ (((h + 1) * _HEAD_MUL) & _MASK64))
    k = _mix64(k ^ (((j + 1) * _ROW_MUL) & _MASK64))
    return k


class _RowStream:
    """Stream of 64-bit words for one (seed, head, query block); word t = mix(key + (t+1)*golden)."""

    def __init__(self, seed: int, h: int, j: int):
        self.key = _row_key(seed, h, j)
        self.ctr = 0

    def word(self) -> int:
        self.ctr += 1
        return _mix64(self.key + self.ctr * _GOLDEN)

    def below(self, m: int) -> int:
        """Unbiased integer in [0, m) by rejection of the incomplete top range."""
        limit = ((1 << 64) // m) * m
        while True:
            u = self.word()
            if u < limit:
                return u % m


def make_rand_idx(H: int, n: int, b: int, g: int, w: int, r: int, seed: int,
                  global_mode: int = GLOBAL_FIRST_LAST) -> np.ndarray:
    """rand_idx[H, nb, r] int32: r distinct random key blocks per (head, query block).

    App. D item 1 ("each query block attends to exactly r random key blocks").
    Candidates are the key blocks outside window(j) and outside G, in ascending
    order; r of them are chosen by a partial Fisher-Yates shuffle driven by the
    row's word stream; the row is stored ascending.  Rows of global query blocks
    are -1 (they attend everything).  Raises if a row has fewer than r candidates.
    """
    if n % b:
        raise ValueError("n must be a multiple of b")
    nb = n // b
    G = set(global_blocks(nb, g, global_mode))
    table = np.full((H, nb, r), -1, dtype=np.int32)
    for h in range(H):
        for j in range(nb):
            if j in G:
                continue
            excluded = G | set(window_blocks(nb, j, w))
            cand = [k for k in range(nb) if k not in excluded]
            if len(cand) < r:
                raise ValueError(f"query block {j}: only {len(cand)} candidates for r={r}")
            stream = _RowStream(seed, h, j)
            for t in range(r):
                i = t + stream.below(len(cand) - t)
                cand[t], cand[i] = cand[i], cand[t]
            table[h, j, :] = sorted(cand[:r])
    return table


def validate_rand_idx(rand_idx: np.ndarray, H: int, n: int, b: int, g: int, w: int, r: int,
                      global_mode: int = GLOBAL_FIRST_LAST) -> bool:
    """True iff every non-global row holds r distinct in-range blocks outside window and G."""
    nb = n // b
    rand_idx = np.asarray(rand_idx)
    if rand_idx.shape != (H, nb, r):
        return False
    G = set(global_blocks(nb, g, global_mode))
    for h in range(H):
        for j in range(nb):
            if j in G:
                continue
            row = [int(x) for x in rand_idx[h, j]]
            excluded = G | set(window_blocks(nb, j, w))
            if len(set(row)) != r:
                return False
            if any(k < 0 or k >= nb or k in excluded for k in row):
                return False
    return True


# --------------------------------------------------------------------------- #
# Neighbour sets and the dense adjacency matrix A (Sec. 2)
# --------------------------------------------------------------------------- #
def neighbour_blocks(rand_idx_h: np.ndarray, nb: int, j: int, g: int, w: int,
                     global_mode: int = GLOBAL_FIRST_LAST) -> list[int]:
    """Sorted key blocks attended by query block j of one head: G u window(j) u random(j).

    A global query block attends every key block (A(i,:) = 1 for i in G, Sec. 2).
    Negative entries of the random table are ignored.
    """
    G = global_blocks(nb, g, global_mode)
    if j in G:
        return list(range(nb))
    s = set(G) | set(window_blocks(nb, j, w))
    if rand_idx_h is not None and rand_idx_h.shape[-1] > 0:
        s |= {int(k) for k in rand_idx_h[j] if 0 <= int(k) < nb}
    return sorted(s)


def dense_block_mask(rand_idx_h: np.ndarray, nb: int, g: int, w: int,
                     global_mode: int = GLOBAL_FIRST_LAST) -> np.ndarray:
    """bool [nb, nb]: entry (j, k) is True iff query block j attends key block k (one head)."""
    M = np.zeros((nb, nb), dtype=bool)
    for j in range(nb):
        M[j, neighbour_blocks(rand_idx_h, nb, j, g, w, global_mode)] = True
    return M


def dense_mask(rand_idx_h: np.ndarray, n: int, b: int, g: int, w: int,
               global_mode: int = GLOBAL_FIRST_LAST) -> np.ndarray:
    """bool [n, n] adjacency matrix A of one head: A(i, k) = block mask(i // b, k // b)."""
    nb = n // b
    Mb = dense_block_mask(rand_idx_h, nb, g, w, global_mode)
    return np.repeat(np.repeat(Mb, b, axis=0), b, axis=1)


def count_block_pairs(rand_idx: np.ndarray, n: int, b: int, g: int, w: int,
                      global_mode: int = GLOBAL_FIRST_LAST,
                      key_block_valid: np.ndarray | None = None,
                      skip_padded_query_blocks: bool = False) -> int:
    """Number of (query block, key block) pairs in the pattern, summed over heads.

    With key_block_valid (bool [nb]) only pairs whose key block holds at least one
    valid key are counted (the useful-work count under a key-padding mask); with
    skip_padded_query_blocks also only those whose query block holds a valid position.
    """
    nb = n // b
    total = 0
    for h in range(rand_idx.shape[0]):
        Mb = dense_block_mask(rand_idx[h], nb, g, w, global_mode)
        if key_block_valid is not None:
            Mb = Mb & np.asarray(key_block_valid, dtype=bool)[None, :]
            if skip_padded_query_blocks:
                Mb = Mb & np.asarray(key_block_valid, dtype=bool)[:, None]
        total += int(Mb.sum())
    return total


def reverse_random_lists(rand_idx_h: np.ndarray, nb: int) -> list[list[int]]:
    """For each key block k, the ascending list of query blocks whose random row holds k."""
    rev: list[list[int]] = [[] for _ in range(nb)]
    for j in range(nb):
        for k in rand_idx_h[j]:
            k = int(k)
            if 0 <= k < nb:
                rev[k].append(j)
    return rev
