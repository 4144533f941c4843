// Host-side integer work on the BigBird block pattern (App. D items 1-3):
// the seeded random-block table, its validator and the block-pair counter.
// No floating point and no device code in this file.
#include "bigbird.h"
#include "pattern_common.h"

#include <algorithm>
#include <vector>

namespace {

// 64-bit finaliser of SplitMix64 (Steele, Lea, Flood: "Fast splittable
// pseudorandom number generators", 2014).
inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kHeadMul = 0xD6E8FEB86659FD93ull;
constexpr uint64_t kRowMul = 0xA0761D6478BD642Full;

// Word stream of one (seed, head, query block): word t = mix(key + (t+1) * golden).
struct RowStream {
  uint64_t key;
  uint64_t ctr = 0;
  RowStream(uint64_t seed, int h, int j) {
    key = mix64(seed + kGolden);
    key = mix64(key ^ (static_cast<uint64_t>(h + 1) * kHeadMul));
    key = mix64(key ^ (static_cast<uint64_t>(j + 1) * kRowMul));
  }
  uint64_t word() { return mix64(key + (++ctr) * kGolden); }
  // Unbiased integer in [0, m): reject words in the incomplete top range.
  uint64_t below(uint64_t m) {
    // floor(2^64 / m) * m, computed without 128-bit arithmetic
    const uint64_t rem = (~m + 1) % m;  // 2^64 mod m
    const uint64_t limit_minus = rem;   // accept u <= 2^64 - 1 - rem
    for (;;) {
      const uint64_t u = word();
      if (u <= ~limit_minus) return u % m;
    }
  }
};

}  // namespace

extern "C" int bigbird_make_rand_idx(int32_t* rand_idx_host, int H, int n, int b, int g, int w,
                                     int r, uint64_t seed, int global_mode) {
  if (!rand_idx_host && H > 0 && r > 0) return BB_ERR_NULL;
  int st = bb::check_pattern_args(H, n, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  const int nb = n / b;
  const bb::Pattern pat{nb, g, w, global_mode};
  std::vector<int32_t> cand;
  cand.reserve(nb);
  for (int h = 0; h < H; ++h) {
    for (int j = 0; j < nb; ++j) {
      int32_t* row = rand_idx_host + (static_cast<size_t>(h) * nb + j) * r;
      if (pat.is_global(j)) {
        std::fill(row, row + r, -1);
        continue;
      }
      cand.clear();
      for (int k = 0; k < nb; ++k)
        if (!pat.is_global(k) && !pat.in_window(j, k)) cand.push_back(k);
      if (static_cast<int>(cand.size()) < r) return BB_ERR_PATTERN;
      RowStream stream(seed, h, j);
      for (int t = 0; t < r; ++t) {
        const uint64_t i = t + stream.below(cand.size() - t);
        std::swap(cand[t], cand[i]);
      }
      std::sort(cand.begin(), cand.begin() + r);
      std::copy(cand.begin(), cand.begin() + r, row);
    }
  }
  return BB_OK;
}

extern "C" int bigbird_validate_rand_idx(const int32_t* rand_idx_host, int H, int n, int b, int g,
                                         int w, int r, int global_mode) {
  if (!rand_idx_host && H > 0 && r > 0) return BB_ERR_NULL;
  int st = bb::check_pattern_args(H, n, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  const int nb = n / b;
  const bb::Pattern pat{nb, g, w, global_mode};
  for (int h = 0; h < H; ++h) {
    for (int j = 0; j < nb; ++j) {
      if (pat.is_global(j)) continue;
      const int32_t* row = rand_idx_host + (static_cast<size_t>(h) * nb + j) * r;
      for (int t = 0; t < r; ++t) {
        const int k = row[t];
        if (k < 0 || k >= nb || pat.is_global(k) || pat.in_window(j, k)) return BB_ERR_PATTERN;
        for (int u = 0; u < t; ++u)
          if (row[u] == k) return BB_ERR_PATTERN;
      }
    }
  }
  return BB_OK;
}

extern "C" int64_t bigbird_count_block_pairs(const int32_t* rand_idx_host,
                                             const uint8_t* key_mask_host, int B, int H, int n,
                                             int b, int g, int w, int r, int global_mode) {
  if (!rand_idx_host && H > 0 && r > 0) return BB_ERR_NULL;
  const bool skip_q = (global_mode & BB_SKIP_PADDED_QUERY_BLOCKS) != 0 && key_mask_host;
  global_mode &= ~BB_SKIP_PADDED_QUERY_BLOCKS;
  int st = bb::check_pattern_args(H, n, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  if (B < 0) return BB_ERR_SHAPE;
  const int nb = n / b;
  const bb::Pattern pat{nb, g, w, global_mode};
  int64_t total = 0;
  std::vector<uint8_t> valid(nb), seen(nb);
  for (int bi = 0; bi < B; ++bi) {
    for (int k = 0; k < nb; ++k) {
      valid[k] = 1;
      if (key_mask_host) {
        valid[k] = 0;
        for (int t = 0; t < b; ++t)
          if (key_mask_host[static_cast<size_t>(bi) * n + static_cast<size_t>(k) * b + t]) valid[k] = 1;
      }
    }
    for (int h = 0; h < H; ++h) {
      for (int j = 0; j < nb; ++j) {
        if (skip_q && !valid[j]) continue;  // a query block without a valid position is not computed
        std::fill(seen.begin(), seen.end(), 0);
        if (pat.is_global(j)) {
          std::fill(seen.begin(), seen.end(), 1);
        } else {
          for (int k = 0; k < nb; ++k)
            if (pat.is_global(k) || pat.in_window(j, k)) seen[k] = 1;
          for (int t = 0; t < r; ++t) {
            const int k = rand_idx_host[(static_cast<size_t>(h) * nb + j) * r + t];
            if (k >= 0 && k < nb) seen[k] = 1;
          }
        }
        for (int k = 0; k < nb; ++k) total += (seen[k] && valid[k]);
      }
    }
  }
  return total;
}
