// Forward kernels: fused S^T = K Q^T -> online softmax -> O^T += V^T P^T per
// (query block, slice of its key-block list), and the merge of sliced rows.
//
// Eq. (AT) of Sec. 2 per head on the blocked pattern of App. D.  Each block pair
// is a dense 64x64x64 contraction, which is what the MFMA units are for.  The
// scores are produced transposed (keys along MFMA rows, queries along MFMA
// columns) so that one lane owns one query column: the row maximum and row sum of
// the softmax are in-lane reductions plus one exchange between the two 32-lane
// halves, and the probabilities sit in registers exactly where the second MFMA
// wants its B operand (the contraction order over keys is free, so V^T is read
// from LDS in the matching permuted key order).
#include "fwd_kernels.h"

#include <cstdio>

namespace bb {

namespace {

template <bool BF16>
struct Tile;

template <>
struct Tile<true> {
  static constexpr int kBytes = kBlk * kDim * 2;  // 8 KB, swizzled 128-byte rows
  static constexpr int kVecPerThread = kBytes / 16 / kThreads;  // 4
};
template <>
struct Tile<false> {
  static constexpr int kBytes = kBlk * kF32Stride * 4;  // 17 KB, padded rows
  static constexpr int kVecPerThread = kBlk * kDim * 4 / 16 / kThreads;  // 8
};

// Global -> registers: one 64x64 tile of K or V, 16 bytes per lane per step, coalesced.
template <bool BF16>
__device__ __forceinline__ void tile_fetch(const void* base, size_t row0, u32x4* regs) {
  const int tid = threadIdx.x;
  constexpr int kRowBytes = BF16 ? 128 : 256;
  constexpr int kChunksPerRow = kRowBytes / 16;
  const char* p = static_cast<const char*>(base) + row0 * kRowBytes;
#pragma unroll
  for (int i = 0; i < Tile<BF16>::kVecPerThread; ++i) {
    const int idx = i * kThreads + tid;
    const int row = idx / kChunksPerRow, c = idx % kChunksPerRow;
    regs[i] = *reinterpret_cast<const u32x4*>(p + row * kRowBytes + c * 16);
  }
}

// Registers -> LDS in the layout the MFMA operand reads expect.
template <bool BF16>
__device__ __forceinline__ void tile_store(char* lds, const u32x4* regs) {
  const int tid = threadIdx.x;
  constexpr int kChunksPerRow = BF16 ? 8 : 16;
#pragma unroll
  for (int i = 0; i < Tile<BF16>::kVecPerThread; ++i) {
    const int idx = i * kThreads + tid;
    const int row = idx / kChunksPerRow, c = idx % kChunksPerRow;
    const int off = BF16 ? tile_off_bf16(row, c) : (row * kF32Stride + c * 4) * 4;
    *reinterpret_cast<u32x4*>(lds + off) = regs[i];
  }
}

}  // namespace

template <bool BF16>
__global__ __launch_bounds__(kThreads) void fwd_kernel(FwdParams p) {
  __shared__ __attribute__((aligned(16))) char lds_k[Tile<BF16>::kBytes];
  __shared__ __attribute__((aligned(16))) char lds_v[Tile<BF16>::kBytes];
  __shared__ int klist[kChunk];

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  WorkItem it;
  if (!decode_item(p.split, pat, p.BH, blockIdx.x, &it)) return;
  const int bi = it.bh / p.H, h = it.bh % p.H;
  const int lane = lane_id(), wv = threadIdx.x >> 6;
  const int hf = lane >> 5, col = lane & 31;

  const int cnt = build_key_list(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, it.j, it.row_global,
                                 it.chunk, klist);
  __syncthreads();

  const size_t bh_row0 = static_cast<size_t>(it.bh) * p.n;       // first row of this (batch, head)
  const size_t qrow = bh_row0 + it.j * kBlk + wv * 32 + col;     // this lane's query row

  // Q^T operand, kept in registers for the whole item.
  bf16x8 qb[4];
  f32x4 qf[8];
  if constexpr (BF16) {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.Q) + qrow * kDim);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qb[ks] = qp[ks * 2 + hf];
  } else {
    const f32x4* qp = reinterpret_cast<const f32x4*>(static_cast<const float*>(p.Q) + qrow * kDim);
#pragma unroll
    for (int u = 0; u < 8; ++u) qf[u] = qp[u * 2 + hf];
  }

  f32x16 o[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_run = neg_inf();  // running maximum of the raw scores q.k (both halves agree)
  float l_run = 0.f;        // this lane's share of the running sum of 2^((q.k - m) c)
  const float c = p.c;

  constexpr int NV = Tile<BF16>::kVecPerThread;
  u32x4 kreg[NV], vreg[NV];
  if (cnt > 0) {
    const size_t krow0 = bh_row0 + static_cast<size_t>(klist[0]) * kBlk;
    tile_fetch<BF16>(p.K, krow0, kreg);
    tile_fetch<BF16>(p.V, krow0, vreg);
  }

  for (int i = 0; i < cnt; ++i) {
    const int kb = klist[i];
    __syncthreads();  // everyone is done reading the previous tiles
    tile_store<BF16>(lds_k, kreg);
    tile_store<BF16>(lds_v, vreg);
    __syncthreads();
    if (i + 1 < cnt) {
      const size_t krow0 = bh_row0 + static_cast<size_t>(klist[i + 1]) * kBlk;
      tile_fetch<BF16>(p.K, krow0, kreg);
      tile_fetch<BF16>(p.V, krow0, vreg);
    }
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, kb);

    // ---- S^T tile: rows = 64 keys (two 32-row MFMA tiles), columns = this wave's 32 queries
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
      const int krow = t * 32 + col;
      if constexpr (BF16) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(lds_k + tile_off_bf16(krow, ks * 2 + hf));
          s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb[ks], s[t], 0, 0, 0);
        }
      } else {
        const float* kr = reinterpret_cast<const float*>(lds_k) + krow * kF32Stride + hf * 4;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const f32x4 a = *reinterpret_cast<const f32x4*>(kr + u * 8);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            s[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], qf[u][e], s[t], 0, 0, 0);
        }
      }
    }

    // ---- padded keys -> -inf (only blocks that are partly padded take this path)
    if (vbits != ~0ull) {
      const uint64_t mine = vbits >> (hf * 4);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!((mine >> (t * 32 + acc_row(r, 0))) & 1)) s[t][r] = neg_inf();
    }

    // ---- online softmax (base 2, scale folded into c)
    float mloc = neg_inf();
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[t][r]);
    mloc = half_max(mloc);
    const float m_new = fmaxf(m_run, mloc);
    const float m_use = (m_new == neg_inf()) ? 0.f : m_new;
    const float alpha = fast_exp2((m_run - m_use) * c);
    const float mc = m_use * c;
    float lsum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = fast_exp2(__builtin_fmaf(s[t][r], c, -mc));
        s[t][r] = pv;
        lsum += pv;
      }
    l_run = l_run * alpha + lsum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;

    // ---- O^T += V^T P^T : rows = d, columns = queries, contraction over the 64 keys
    if constexpr (BF16) {
      bf16x8 pb[4];
#pragma unroll
      for (int sgrp = 0; sgrp < 4; ++sgrp)
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
          pb[sgrp][kk] = static_cast<__bf16>(s[sgrp >> 1][(sgrp & 1) * 8 + kk]);
      // Transposing LDS read: inside a 16-lane group lane i addresses 4 values of
      // row i/4 and receives, for its own column, the values of rows 0..3.
      const int gq = lane >> 4, li = lane & 15;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const int chunk = dt * 4 + (gq & 1) * 2 + ((li & 3) >> 1);
        const int sub = (li & 1) * 8;
#pragma unroll
        for (int sgrp = 0; sgrp < 4; ++sgrp) {
          const int row1 = sgrp * 16 + hf * 4 + (li >> 2);
          const int row2 = row1 + 8;
          const s16x4 lo = lds_read_tr16(lds_v + tile_off_bf16(row1, chunk) + sub);
          const s16x4 hi = lds_read_tr16(lds_v + tile_off_bf16(row2, chunk) + sub);
          union { struct { s16x4 a, b; } h2; bf16x8 v; } a;
          a.h2.a = lo;
          a.h2.b = hi;
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pb[sgrp], o[dt], 0, 0, 0);
        }
      }
    } else {
      const float* vbase = reinterpret_cast<const float*>(lds_v);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = t * 32 + acc_row(r, hf);
            const float a = vbase[key * kF32Stride + dt * 32 + col];
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, s[t][r], o[dt], 0, 0, 0);
          }
    }
  }

  // ---- finalise: O = O~ / l, LSE = m*scale + ln l   (or hand the partial triple on)
  const float l_tot = half_sum(l_run);
  const int qi = wv * 32 + col;  // query row inside the block
  if (it.nchunks == 1) {
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (hf == 0)
      p.LSE[qrow] = l_tot > 0.f ? (m_run * c + fast_log2(l_tot)) * kLn2 : neg_inf();
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d0 = dt * 32 + acc_row(r4 * 4, hf);
        if constexpr (BF16) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[dt][r4 * 4 + e] * inv);
          *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.O) + qrow * kDim + d0) = v;
        } else {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[dt][r4 * 4 + e] * inv;
          *reinterpret_cast<f32x4*>(static_cast<float*>(p.O) + qrow * kDim + d0) = v;
        }
      }
  } else {
    float* po = p.part_o + static_cast<size_t>(it.slot) * (kBlk * kDim);
    float* pml = p.part_ml + static_cast<size_t>(it.slot) * (2 * kBlk);
    if (hf == 0) {
      pml[qi] = (m_run == neg_inf()) ? neg_inf() : m_run * c;
      pml[kBlk + qi] = l_tot;
    }
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d0 = dt * 32 + acc_row(r4 * 4, hf);
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = o[dt][r4 * 4 + e];
        *reinterpret_cast<f32x4*>(po + qi * kDim + d0) = v;
      }
  }
}

// Merge the slices of a split row: M = max m_c, L = sum l_c 2^(m_c - M),
// O = sum O~_c 2^(m_c - M) / L, LSE = (M + log2 L) ln 2.  One workgroup per
// (batch, head, split row); thread t owns query t/4 and 16 of its d columns.
template <bool BF16>
__global__ __launch_bounds__(256) void fwd_combine_kernel(FwdParams p) {
  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const RowSplit& s = p.split;
  const int nglob_rows = s.cg > 1 ? p.g : 0;
  const int nsparse_rows = s.cs > 1 ? p.nb - p.g : 0;
  const int rows_per_bh = nglob_rows + nsparse_rows;
  const int bh = blockIdx.x / rows_per_bh, rr = blockIdx.x % rows_per_bh;
  int j, nchunks, slot0;
  if (rr < nglob_rows) {
    j = pat.global_block(rr);
    nchunks = s.cg;
    slot0 = bh * s.slots_per_bh + rr * s.cg;
  } else {
    const int t = rr - nglob_rows;
    j = pat.sparse_block(t);
    nchunks = s.cs;
    slot0 = bh * s.slots_per_bh + (s.cg > 1 ? p.g * s.cg : 0) + t * s.cs;
  }
  const int q = threadIdx.x >> 2, d0 = (threadIdx.x & 3) * 16;
  float M = neg_inf();
  for (int cidx = 0; cidx < nchunks; ++cidx)
    M = fmaxf(M, p.part_ml[static_cast<size_t>(slot0 + cidx) * (2 * kBlk) + q]);
  float acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  float L = 0.f;
  if (M != neg_inf()) {
    for (int cidx = 0; cidx < nchunks; ++cidx) {
      const float* pml = p.part_ml + static_cast<size_t>(slot0 + cidx) * (2 * kBlk);
      const float mcur = pml[q];
      if (mcur == neg_inf()) continue;
      const float wgt = fast_exp2(mcur - M);
      L += pml[kBlk + q] * wgt;
      const f32x4* po = reinterpret_cast<const f32x4*>(
          p.part_o + static_cast<size_t>(slot0 + cidx) * (kBlk * kDim) + q * kDim + d0);
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        const f32x4 v = po[v4];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[v4 * 4 + e] += v[e] * wgt;
      }
    }
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  const size_t row = static_cast<size_t>(bh) * p.n + j * kBlk + q;
  if ((threadIdx.x & 3) == 0) p.LSE[row] = L > 0.f ? (M + fast_log2(L)) * kLn2 : neg_inf();
  if constexpr (BF16) {
    bf16x8 v0, v1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      v0[e] = static_cast<__bf16>(acc[e] * inv);
      v1[e] = static_cast<__bf16>(acc[8 + e] * inv);
    }
    bf16x8* dst = reinterpret_cast<bf16x8*>(static_cast<__bf16*>(p.O) + row * kDim + d0);
    dst[0] = v0;
    dst[1] = v1;
  } else {
    f32x4* dst = reinterpret_cast<f32x4*>(static_cast<float*>(p.O) + row * kDim + d0);
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = acc[v4 * 4 + e] * inv;
      dst[v4] = v;
    }
  }
}

namespace {
// Reports a failed launch on stderr (the status code cannot carry the runtime's reason).
bool launch_failed(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return false;
  fprintf(stderr, "bigbird: launch of %s failed: %s\n", what, hipGetErrorString(e));
  return true;
}
}  // namespace

int launch_fwd(const FwdParams& p, bool bf16, hipStream_t stream) {
  const RowSplit& s = p.split;
  const unsigned grid = static_cast<unsigned>(kXcd) * s.bh_rounds * s.items_per_bh;
  if (grid == 0) return BB_OK;
  if (bf16)
    hipLaunchKernelGGL(fwd_kernel<true>, dim3(grid), dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL(fwd_kernel<false>, dim3(grid), dim3(kThreads), 0, stream, p);
  if (launch_failed("fwd_kernel")) return BB_ERR_LAUNCH;
  const int rows_per_bh = (s.cg > 1 ? p.g : 0) + (s.cs > 1 ? p.nb - p.g : 0);
  if (rows_per_bh > 0) {
    const unsigned cgrid = static_cast<unsigned>(p.BH) * rows_per_bh;
    if (bf16)
      hipLaunchKernelGGL(fwd_combine_kernel<true>, dim3(cgrid), dim3(256), 0, stream, p);
    else
      hipLaunchKernelGGL(fwd_combine_kernel<false>, dim3(cgrid), dim3(256), 0, stream, p);
    if (launch_failed("fwd_combine_kernel")) return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
