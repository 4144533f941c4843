// Attention dropout: the keep mask as a function of (seed, batch*H + head, query, key).
//
// The paper names only the rate (App. E.1: "attention dropout 0.1").  Here an attended
// probability P_ij is kept with probability 1 - p and the kept ones are scaled by 1 / (1 - p);
// LSE stays that of the undropped softmax.  The mask must be the same in the forward and in both
// backward kernels, whatever their tiling, so it is computed from the element's coordinates by a
// counter-based generator on 32-bit integers (arithmetic modulo 2^32):
//   mix(x):  x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16
//   row key  rk(i)   = mix(seed_lo ^ mix(seed_hi ^ (bh * n + i)))
//   word     w(i, j) = mix(rk(i) ^ ((j >> 1) * 0x9E3779B9))      -- one word per pair of keys
//   number   u(i, j) = bits 0..14 of w for even j, bits 16..30 for odd j
//   keep     u(i, j) >= T,  T = round(p * 32768)
// so the rate realised is T / 32768 and the scale 32768 / (32768 - T).  A row key costs two
// mixes per (query, work item); a word serves the two keys that share a packed bf16 register in
// the kernels whose lanes own a query.
#ifndef BB_DROPOUT_H_
#define BB_DROPOUT_H_

#include <stdint.h>

#include "pattern_common.h"

namespace bb {

struct Dropout {
  uint32_t thr;      // T; 0 = no dropout
  uint32_t seed_lo, seed_hi;
  float rs;          // 32768 / (32768 - T); 1 without dropout
};

BB_HD uint32_t drop_mix(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

// rowid = (batch*H + head) * n + query, as a 32-bit number
BB_HD uint32_t drop_row_key(const Dropout& dr, uint32_t rowid) {
  return drop_mix(dr.seed_lo ^ drop_mix(dr.seed_hi ^ rowid));
}

// the word of keys 2*pair and 2*pair + 1
BB_HD uint32_t drop_word(uint32_t rk, uint32_t pair) { return drop_mix(rk ^ (pair * 0x9E3779B9u)); }

BB_HD bool drop_keep_even(uint32_t w, uint32_t thr) { return (w & 0x7fffu) >= thr; }
BB_HD bool drop_keep_odd(uint32_t w, uint32_t thr) { return ((w >> 16) & 0x7fffu) >= thr; }

BB_HD bool drop_keep(const Dropout& dr, uint32_t rowid, uint32_t key) {
  const uint32_t w = drop_word(drop_row_key(dr, rowid), key >> 1);
  return (key & 1u) ? drop_keep_odd(w, dr.thr) : drop_keep_even(w, dr.thr);
}

// Host: rate and seed -> parameters.  False if p is not in [0, 1) or rounds to 1.
inline bool make_dropout(float p, uint64_t seed, Dropout* out) {
  if (!(p >= 0.f) || !(p < 1.f)) return false;
  const uint32_t t = static_cast<uint32_t>(static_cast<double>(p) * 32768.0 + 0.5);
  if (t >= 32768u) return false;
  out->thr = t;
  out->seed_lo = static_cast<uint32_t>(seed);
  out->seed_hi = static_cast<uint32_t>(seed >> 32);
  out->rs = static_cast<float>(32768.0 / (32768.0 - static_cast<double>(t)));
  return true;
}

}  // namespace bb
#endif  // BB_DROPOUT_H_
