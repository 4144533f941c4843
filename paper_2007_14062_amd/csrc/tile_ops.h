// Asynchronous tile staging and synchronisation pieces shared by the bf16 kernels.
#ifndef BB_TILE_OPS_H_
#define BB_TILE_OPS_H_

#include "kernel_common.h"

namespace bb {

// s_waitcnt immediate that waits for all but `n` vector-memory loads (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, other counters left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
constexpr int kLgkmcnt0 = 15 | (3 << 14) | (7 << 4);  // wait for all LDS reads, nothing else

// Enqueue this wave's half of a 64x64 bf16 tile: global -> LDS, 16 bytes per lane,
// four instructions per wave.  Instruction ii of wave wv fills LDS rows
// 8*(2*ii+wv) .. +8 linearly (the hardware places lane l at M0 + 16*l), so the XOR
// swizzle is applied on the global side: the lane that lands on chunk position p of
// row r fetches chunk p ^ tile_swizzle(r).  `voff` is that per-lane byte offset inside
// the tile (tile_load_lane_offset, fixed for the kernel), `gtile` the wave-uniform tile
// address, `lds` the LDS byte address of this wave's first 1 KB slot.
// Written as inline asm so that the compiler's wait-count bookkeeping does not see
// these loads: it would otherwise drain them before every LDS read.  The waits
// are placed by hand (loads return in order, so vmcnt(N) is exact).
__device__ __forceinline__ void tile_load_async(const char* gtile, unsigned lds, unsigned voff) {
  // the instruction offset moves the global and the LDS address alike: two base pairs per tile
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 4\n\t"  // wait states the compiler cannot see to from outside: M0 written by a scalar instruction (1) and an
                       // address register pair that a vector instruction (v_readlane) may just have written (5)
        "global_load_lds_dwordx4 %0, %1\n\t"
        "global_load_lds_dwordx4 %0, %1 offset:2048"
        :
        : "v"(voff), "s"(gtile + hh * 4096), "s"(lds + hh * 4096)
        : "memory");  // M0 is written here; nothing else in this kernel reads M0
}

__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return static_cast<unsigned>(reinterpret_cast<uintptr_t>((BB_LDS const char*)(p)));
}


// Enqueue one 256-byte vector (64 floats): global -> LDS, 4 bytes per lane, lane l
// lands at lds + 4*l.  `gvec` is the wave-uniform address of the vector.
__device__ __forceinline__ void vec_load_async(const float* gvec, unsigned lds, unsigned lane) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 4\n\t"
      "global_load_lds_dword %0, %1"
      :
      : "v"(lane * 4u), "s"(gvec), "s"(lds)
      : "memory");
}

// MFMA operand fragments of a 64x64 bf16 tile held in LDS (128-byte rows, swizzled
// chunks).  "Straight": the tile's rows are the MFMA's non-contracted index and its
// columns (d) the contraction: fragment [t][ks] = row 32t + lane%32, columns
// 16ks + 8*(lane/32) .. +8.  Used for K in S^T = K Q^T, for V in dP^T = V dO^T, for Q
// and dO in the key-major backward kernel.
struct StraightOffsets {
  int off[4];  // byte offsets for ks = 0..3 of row lane%32 (t adds 4096)
  __device__ __forceinline__ explicit StraightOffsets(int lane) {
    const int col = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) off[ks] = tile_off_bf16(col, ks * 2 + hf);
  }
  __device__ __forceinline__ void read(const char* tile, bf16x8 (&f)[2][4]) const {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        f[t][ks] = *reinterpret_cast<const bf16x8*>(tile + off[ks] + t * 4096);
  }
};

// "Transposed": the tile's rows are the contraction index, taken in the order the
// 32x32 accumulator layout hands them over: fragment [dt][sg] belongs to output row
// (tile column) 32dt + lane%32 and holds, in contraction slot 8*(lane/32) + kk, tile
// row 16sg + 4*(lane/32) + kk (kk < 4) or 16sg + 8 + 4*(lane/32) + kk - 4.  Read with
// ds_read_b64_tr_b16.  Used for V^T in O^T += V^T P^T, K^T in dQ^T += K^T dS^T, dO^T and
// Q^T in the key-major backward kernel.
struct TransposedOffsets {
  int off[2][2];  // byte offsets for dt = 0, 1 and the two 4-row pieces (sg adds 2048)
  __device__ __forceinline__ explicit TransposedOffsets(int lane) {
    const int hf = lane >> 5, gq = lane >> 4, li = lane & 15;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int half = 0; half < 2; ++half)
        off[dt][half] = tile_off_bf16(half * 8 + hf * 4 + (li >> 2), dt * 4 + (gq & 1) * 2 + ((li & 3) >> 1)) +
                        (li & 1) * 8;
  }
  __device__ __forceinline__ bf16x8 read_one(const char* tile, int dt, int sg) const {
    // rows 16*sg + {0, 8} + (4*hf + li/4): adding a multiple of 16 rows keeps the swizzle
    const s16x4 lo = lds_read_tr16(tile + off[dt][0] + sg * 2048);
    const s16x4 hi = lds_read_tr16(tile + off[dt][1] + sg * 2048);
    union { struct { s16x4 a, b; } h2; bf16x8 v; } u;
    u.h2.a = lo;
    u.h2.b = hi;
    return u.v;
  }
  __device__ __forceinline__ void read(const char* tile, bf16x8 (&f)[2][4]) const {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) f[dt][sg] = read_one(tile, dt, sg);
  }
};

// Accumulator tile pair [2][16] (rows 64 x this lane's column) -> the four bf16 B-operand
// fragments of the next MFMA (slot order as in TransposedOffsets).
__device__ __forceinline__ void pack_acc_bf16(const f32x16 (&a)[2], bf16x8 (&b)[4]) {
#pragma unroll
  for (int sg = 0; sg < 4; ++sg)
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) b[sg][kk] = static_cast<__bf16>(a[sg >> 1][(sg & 1) * 8 + kk]);
}

}  // namespace bb

// Workgroup barrier without the memory fence of __syncthreads(): the fence would
// drain the LDS-bound loads still in flight.  Ordering is kept by the explicit
// counter waits next to each use; the empty asm stops compiler reordering.
#define BB_BARRIER()                       \
  do {                                     \
    asm volatile("" ::: "memory");         \
    __builtin_amdgcn_s_barrier();          \
    asm volatile("" ::: "memory");         \
  } while (0)


#endif  // BB_TILE_OPS_H_
