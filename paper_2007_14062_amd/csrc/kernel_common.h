// Device-side helpers shared by the forward and backward kernels (gfx950 only).
#ifndef BB_KERNEL_COMMON_H_
#define BB_KERNEL_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pattern_common.h"

namespace bb {

constexpr int kBlk = 64;      // block length b (App. E.1: 64 for every ITC model)
constexpr int kDim = 64;      // head width d
constexpr int kChunk = 8;     // list entries per slice of a global row / global key column
constexpr int kSparseChunk = 16;  // most key blocks per work item of a non-global row (the ITC base pattern has g+w+r = 8)
constexpr int kChunkGlobal = 8;  // key blocks per work item of a global row (equal to kChunk; 16 measured the same backward time)
constexpr int kChunkMax = kChunkGlobal > kSparseChunk ? kChunkGlobal : kSparseChunk;
constexpr int kWaves = 2;     // one wave owns 32 query rows of the 64-row block
constexpr int kThreads = 64 * kWaves;
constexpr int kXcd = 8;       // accelerator dies; workgroup id modulo 8 selects the die
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

#define BB_LDS __attribute__((address_space(3)))

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

// v_exp_f32: 2^x, flushes tiny results to zero; arguments here are <= 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Value of x in the other 32-lane half of the wave, combined with max / add.
__device__ __forceinline__ float half_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Rank of this lane among the set bits of a wave-wide mask (number of set bits below it).
__device__ __forceinline__ int mask_rank(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0));
}

// Register-index -> row mapping of a 32x32 MFMA accumulator: element r of lane l
// sits in row 8*(r/4) + 4*(l/32) + r%4, column l%32.
__device__ __forceinline__ constexpr int acc_row(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

// Bank swizzle of a 64x64 bf16 tile kept in LDS with 128-byte rows: 16-byte chunk c of
// row `row` is stored at chunk position c ^ tile_swizzle(row).  LDS has 64 four-byte
// banks, so the row parity already selects a bank half and the swizzle uses row bits
// 1..3: bit 1 goes to position bit 2 (two rows of equal parity read by one transposing
// load then use different 64-byte halves), bits 2..3 to position bits 0..1 (the eight
// equal-parity rows read by one 16-lane pass of a 128-bit load get eight positions).
__device__ __forceinline__ int tile_swizzle(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }

// Byte offset of 16-byte chunk c of row `row` in such a tile.
__device__ __forceinline__ int tile_off_bf16(int row, int chunk) {
  return row * 128 + ((chunk ^ tile_swizzle(row)) << 4);
}

// Per-lane byte offset inside a tile for the asynchronous tile loads: instruction ii of
// wave wv fills rows 16*ii + 8*wv .. +8 linearly, lane l landing on row l/8, chunk
// position l%8, so it must fetch the chunk that the swizzle stores there.
__device__ __forceinline__ unsigned tile_load_lane_offset(int wv, int lane) {
  const int row = wv * 8 + (lane >> 3);  // + 16*ii: bits 1..3 of the row do not depend on ii
  return row * 128 + (((lane & 7) ^ tile_swizzle(row)) << 4);
}

// ds_read_b64_tr_b16: inside each group of 16 lanes, lane i passes the address of
// four 16-bit values (a piece of matrix row i/4, columns 4*(i%4)..+3) and gets back
// the four rows' values of column i -- a 4x16 block read transposed.
__device__ __forceinline__ s16x4 lds_read_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((BB_LDS s16x4*)(p));
}

constexpr int kF32Stride = 68;  // floats per row of an fp32 tile in LDS (64 + 4 padding)

// Decoded work item: which query block and which slice of its key-block list.
struct WorkItem {
  int bh;       // batch * H + head
  int j;        // query block
  int chunk;    // slice number: entries [chunk*len, (chunk+1)*len) of the row's key-block list,
                // len = kChunkGlobal for a global row, kSparseChunk otherwise
  int nchunks;  // slices this row is split into
  int slot;     // partial-result slot (valid when nchunks > 1)
  bool row_global;
};

// Launch geometry shared by forward and dQ: rows of global query blocks are split
// into cg slices, other rows into cs slices; global rows come first (longest first).
struct RowSplit {
  int cg, cs;         // slices per global / per non-global row
  int items_per_bh;   // g*cg + (nb-g)*cs
  int slots_per_bh;   // partial slots: (cg>1 ? g*cg : 0) + (cs>1 ? (nb-g)*cs : 0)
  int bh_rounds;      // ceil(B*H / 8)
};

inline RowSplit make_row_split(int BH, int nb, int g, int w, int r) {
  RowSplit s;
  int sparse_ub = g + w + r;
  if (sparse_ub > nb) sparse_ub = nb;
  s.cg = (nb + kChunkGlobal - 1) / kChunkGlobal;
  s.cs = (sparse_ub + kSparseChunk - 1) / kSparseChunk;
  if (s.cs < 1) s.cs = 1;
  s.items_per_bh = g * s.cg + (nb - g) * s.cs;
  s.slots_per_bh = (s.cg > 1 ? g * s.cg : 0) + (s.cs > 1 ? (nb - g) * s.cs : 0);
  s.bh_rounds = (BH + kXcd - 1) / kXcd;
  return s;
}

// Workgroup id -> work item.  Hardware hands consecutive workgroup ids to the 8
// dies round robin, so id % 8 picks the die and all items of one (batch, head)
// are given to one die: its K and V (1 MB at n = 4096) stay in that die's L2.
__device__ __forceinline__ bool decode_item(const RowSplit& s, const Pattern& pat, int BH,
                                            unsigned wg, WorkItem* it) {
  const int xcd = wg % kXcd;
  const unsigned q = wg / kXcd;
  const int round = q / s.items_per_bh;
  const int item = q % s.items_per_bh;
  it->bh = round * kXcd + xcd;
  if (it->bh >= BH) return false;
  const int nglob = pat.g * s.cg;
  if (item < nglob) {
    it->row_global = true;
    it->j = pat.global_block(item / s.cg);
    it->chunk = item % s.cg;
    it->nchunks = s.cg;
    it->slot = it->bh * s.slots_per_bh + item;
  } else {
    const int t = item - nglob;
    it->row_global = false;
    it->j = pat.sparse_block(t / s.cs);
    it->chunk = t % s.cs;
    it->nchunks = s.cs;
    it->slot = it->bh * s.slots_per_bh + (s.cg > 1 ? nglob : 0) + t;
  }
  return true;
}

// Does key block k of batch bi hold at least one valid key?  (64 mask bytes)
__device__ __forceinline__ bool block_has_valid_key(const uint8_t* kmask, int bi, int n, int k) {
  const u32x4* p = reinterpret_cast<const u32x4*>(kmask + static_cast<size_t>(bi) * n + k * kBlk);
  unsigned any = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    u32x4 v = p[i];
    any |= v[0] | v[1] | v[2] | v[3];
  }
  return any != 0;
}

// The 64 mask bytes of key block k of batch bi (a byte is a flag): is any key valid, is any padded?
__device__ __forceinline__ void block_mask_flags(const uint8_t* kmask, int bi, int n, int k, bool& any_valid,
                                                 bool& any_padded) {
  const u32x4* p = reinterpret_cast<const u32x4*>(kmask + static_cast<size_t>(bi) * n + k * kBlk);
  unsigned any = 0, zero_byte = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const u32x4 v = p[i];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      any |= v[e];
      zero_byte |= (v[e] - 0x01010101u) & ~v[e] & 0x80808080u;  // some byte of v[e] is 0
    }
  }
  any_valid = any != 0;
  any_padded = zero_byte != 0;
}

// Key blocks attended by query block j of head h (App. D items 1-3 as a set
// union, minus blocks without a valid key), slice `chunk` (see WorkItem) of the
// ascending-by-candidate list: entries [lo, lo+len).  Every lane of the calling wave takes
// part; the slice is written to klist[0..count) and the count returned (wave uniform).
// Candidate order: global blocks, window blocks, random blocks; a candidate is
// dropped if an earlier component already holds it.
__device__ __forceinline__ int build_key_list_range(const Pattern& pat, const int32_t* rand_idx, int r,
                                                    const uint8_t* kmask, int n, int bi, int h, int j,
                                                    bool row_global, int lo, int len, int* klist) {
  const int lane = lane_id();
  const int nb = pat.nb;
  const int ncand = row_global ? nb : pat.g + pat.w + r;
  const int hi = lo + len;
  const int32_t* rrow = rand_idx ? rand_idx + (static_cast<size_t>(h) * nb + j) * r : nullptr;
  int base = 0;
  for (int c0 = 0; c0 < ncand && base < hi; c0 += 64) {
    const int ci = c0 + lane;
    bool valid = false;
    int k = -1;
    if (ci < ncand) {
      if (row_global) {
        k = ci;
        valid = true;
      } else if (ci < pat.g) {
        k = pat.global_block(ci);
        valid = true;
      } else if (ci < pat.g + pat.w) {
        k = j - pat.half() + (ci - pat.g);
        valid = k >= 0 && k < nb && !pat.is_global(k);
      } else if (rrow) {
        const int t = ci - pat.g - pat.w;
        k = rrow[t];
        valid = k >= 0 && k < nb && !pat.is_global(k) && !pat.in_window(j, k);
        for (int u = 0; u < t && valid; ++u) valid = rrow[u] != k;
      }
      if (valid && kmask) valid = block_has_valid_key(kmask, bi, n, k);
    }
    const uint64_t m = __ballot(valid);
    const int rank = base + mask_rank(m);
    if (valid && rank >= lo && rank < hi) klist[rank - lo] = k;
    base += __popcll(m);
  }
  int cnt = base - lo;
  cnt = cnt < 0 ? 0 : (cnt > len ? len : cnt);
  return cnt;
}

// The same with the slice given by its number (see WorkItem).
__device__ __forceinline__ int build_key_list(const Pattern& pat, const int32_t* rand_idx, int r,
                                              const uint8_t* kmask, int n, int bi, int h, int j,
                                              bool row_global, int chunk, int* klist) {
  const int len = row_global ? kChunkGlobal : kSparseChunk;
  return build_key_list_range(pat, rand_idx, r, kmask, n, bi, h, j, row_global, chunk * len, len, klist);
}

// 64-bit validity mask of the keys of block k (bit t = key k*64+t is valid).
__device__ __forceinline__ uint64_t key_valid_bits(const uint8_t* kmask, int bi, int n, int k) {
  const uint8_t v = kmask[static_cast<size_t>(bi) * n + k * kBlk + lane_id()];
  return __ballot(v != 0);
}

}  // namespace bb
#endif  // BB_KERNEL_COMMON_H_
