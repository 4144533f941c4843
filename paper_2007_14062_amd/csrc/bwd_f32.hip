// Backward kernels, fp32 end to end: the correctness configuration of the backward pass
// (plain vector arithmetic, no matrix instructions, not tuned).  Same calculus as the
// bf16 kernels (eq. (AT) of Sec. 2 differentiated on the blocked pattern of App. D):
//   dV = P^T dO;  dP = dO V^T;  D_i = sum_c dO_ic O_ic;  dS = P o (dP - D);
//   dQ = scale dS K;  dK = scale dS^T Q,
// with P recomputed from Q, K and the forward's LSE.  No atomics and no partial results:
// one workgroup owns one query block (dQ) or one key block (dK, dV) and walks its whole
// list, so the summation order is fixed.
#include "bwd_kernels.h"

#include <cstdio>

namespace bb {

namespace {

constexpr int kF32Threads = 256;
constexpr int kTileStride = kDim + 4;  // floats per LDS row of a [64][64] tile: 16-byte rows, shifted banks
constexpr int kListChunk = 64;         // list entries built at a time

// [64][64] fp32 rows from global memory into an LDS tile, by the whole workgroup.
__device__ __forceinline__ void load_tile_f32(const float* src, float* dst) {
  for (int e = threadIdx.x; e < kBlk * kDim / 4; e += kF32Threads) {
    const int row = e >> 4, c4 = e & 15;
    *reinterpret_cast<f32x4*>(dst + row * kTileStride + c4 * 4) =
        *reinterpret_cast<const f32x4*>(src + row * kDim + c4 * 4);
  }
}

__device__ __forceinline__ float dot_row(const float (&a)[kDim], const float* row) {
  float s = 0.f;
#pragma unroll
  for (int c4 = 0; c4 < kDim / 4; ++c4) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(row + c4 * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) s = __builtin_fmaf(a[c4 * 4 + e], v[e], s);
  }
  return s;
}

}  // namespace

// ---------------------------------------------------------------------------------------
// dQ (and the row sums D): one workgroup per (batch*head, query block).  Thread t: query
// t % 64 of the block, keys 16 (t / 64) .. + 15 of every key block of the row's list.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kF32Threads) void bwd_f32_dq_kernel(BwdParams p) {
  __shared__ __attribute__((aligned(16))) float lds_k[kBlk * kTileStride];
  __shared__ __attribute__((aligned(16))) float lds_v[kBlk * kTileStride];
  __shared__ __attribute__((aligned(16))) float lds_red[kBlk * (kDim + 1)];
  __shared__ int klist[kListChunk];
  __shared__ int kcount;

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const int bh = blockIdx.x / p.nb, j = blockIdx.x % p.nb;
  const int bi = bh / p.H, h = bh % p.H;
  const int i = threadIdx.x & 63, kg = threadIdx.x >> 6;
  const size_t bh_row0 = static_cast<size_t>(bh) * p.n;
  const size_t qrow = bh_row0 + static_cast<size_t>(j) * kBlk + i;
  const float* Q = static_cast<const float*>(p.Q);
  const float* K = static_cast<const float*>(p.K);
  const float* V = static_cast<const float*>(p.V);
  const float* O = static_cast<const float*>(p.O);
  const float* dO = static_cast<const float*>(p.dO);

  float q[kDim], go[kDim], dq[kDim];
  float dsum = 0.f;
#pragma unroll
  for (int c4 = 0; c4 < kDim / 4; ++c4) {
    const f32x4 qv = *reinterpret_cast<const f32x4*>(Q + qrow * kDim + c4 * 4);
    const f32x4 gv = *reinterpret_cast<const f32x4*>(dO + qrow * kDim + c4 * 4);
    const f32x4 ov = *reinterpret_cast<const f32x4*>(O + qrow * kDim + c4 * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      q[c4 * 4 + e] = qv[e];
      go[c4 * 4 + e] = gv[e];
      dq[c4 * 4 + e] = 0.f;
      dsum = __builtin_fmaf(gv[e], ov[e], dsum);
    }
  }
  // a query block that was skipped (no valid position) behaves like rows without a valid key
  const bool skip = p.skip_q && !block_has_valid_key(p.kmask, bi, p.n, j);
  if (skip) dsum = 0.f;
  const float lse = p.LSE[qrow];
  const float lse2 = (skip || lse == neg_inf()) ? __builtin_inff() : lse * kLog2e;  // no valid key: every P is 0
  if (kg == 0) {
    p.Dvec[qrow] = dsum;
    p.Lvec[qrow] = lse2;
  }
  const float c = p.c;
  const bool row_global = pat.is_global(j);
  // attention dropout: dP = M / (1 - p) o (dO V^T), M this row of the keep mask
  const uint32_t drop_rk = p.drop.thr ? drop_row_key(p.drop, static_cast<uint32_t>(qrow)) : 0u;

  for (int lo = 0;; lo += kListChunk) {
    __syncthreads();  // the previous chunk's list and tiles are no longer read
    if (threadIdx.x < 64) {
      const int cnt = build_key_list_range(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, j, row_global, lo,
                                           kListChunk, klist);
      if (threadIdx.x == 0) kcount = cnt;
    }
    __syncthreads();
    const int cnt = kcount;
    for (int u = 0; u < cnt; ++u) {
      const int kb = klist[u];
      __syncthreads();  // tiles of the previous key block are no longer read
      load_tile_f32(K + (bh_row0 + static_cast<size_t>(kb) * kBlk) * kDim, lds_k);
      load_tile_f32(V + (bh_row0 + static_cast<size_t>(kb) * kBlk) * kDim, lds_v);
      __syncthreads();
      for (int t = 0; t < 16; ++t) {
        const int kk = kg * 16 + t;
        const bool valid = !p.kmask || p.kmask[static_cast<size_t>(bi) * p.n + kb * kBlk + kk] != 0;
        const float* krow = lds_k + kk * kTileStride;
        const float s = dot_row(q, krow);
        float dp = dot_row(go, lds_v + kk * kTileStride);
        if (p.drop.thr) {
          const uint32_t key = static_cast<uint32_t>(kb * kBlk + kk);
          const uint32_t wd = drop_word(drop_rk, key >> 1);
          const bool keep = (key & 1u) ? drop_keep_odd(wd, p.drop.thr) : drop_keep_even(wd, p.drop.thr);
          dp = keep ? dp * p.drop.rs : 0.f;
        }
        const float pr = valid ? fast_exp2(__builtin_fmaf(s, c, -lse2)) : 0.f;
        const float ds = pr * (dp - dsum);
#pragma unroll
        for (int c4 = 0; c4 < kDim / 4; ++c4) {
          const f32x4 kv = *reinterpret_cast<const f32x4*>(krow + c4 * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) dq[c4 * 4 + e] = __builtin_fmaf(ds, kv[e], dq[c4 * 4 + e]);
        }
      }
    }
    if (cnt < kListChunk) break;
  }

  // the four key groups' shares of dQ, added in group order
  for (int gsrc = 1; gsrc < 4; ++gsrc) {
    __syncthreads();
    if (kg == gsrc)
#pragma unroll
      for (int d = 0; d < kDim; ++d) lds_red[i * (kDim + 1) + d] = dq[d];
    __syncthreads();
    if (kg == 0)
#pragma unroll
      for (int d = 0; d < kDim; ++d) dq[d] += lds_red[i * (kDim + 1) + d];
  }
  if (kg == 0) {
#pragma unroll
    for (int c4 = 0; c4 < kDim / 4; ++c4) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = dq[c4 * 4 + e] * p.scale;
      *reinterpret_cast<f32x4*>(p.dQ + qrow * kDim + c4 * 4) = v;
    }
  }
}

// ---------------------------------------------------------------------------------------
// dK, dV: one workgroup per (batch*head, key block k), over every query block that attends k
// (the inverse of the pattern: every block if k is global; else the global query blocks, the
// window and the rows of rand_idx that name k).  Per query block, first thread t computes
// P and dS for key t % 64 and queries 16 (t / 64) .. + 15 into LDS, then thread t adds the
// products into d columns 16 (t / 64) .. + 15 of key t % 64.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kF32Threads) void bwd_f32_dkv_kernel(BwdParams p) {
  __shared__ __attribute__((aligned(16))) float lds_q[kBlk * kTileStride];
  __shared__ __attribute__((aligned(16))) float lds_do[kBlk * kTileStride];
  __shared__ float lds_p[kBlk * (kBlk + 1)];   // [query][key]
  __shared__ float lds_ds[kBlk * (kBlk + 1)];
  __shared__ float lds_lse[kBlk], lds_d[kBlk];
  __shared__ int jlist[kListChunk];
  __shared__ int jcount;

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const int nb = p.nb;
  const int bh = blockIdx.x / nb, k = blockIdx.x % nb;
  const int bi = bh / p.H, h = bh % p.H;
  const int kk = threadIdx.x & 63, part = threadIdx.x >> 6;
  const size_t bh_row0 = static_cast<size_t>(bh) * p.n;
  const size_t krow = bh_row0 + static_cast<size_t>(k) * kBlk + kk;
  const float* Q = static_cast<const float*>(p.Q);
  const float* K = static_cast<const float*>(p.K);
  const float* V = static_cast<const float*>(p.V);
  const float* dO = static_cast<const float*>(p.dO);

  float kr[kDim], vr[kDim];
#pragma unroll
  for (int c4 = 0; c4 < kDim / 4; ++c4) {
    const f32x4 kv = *reinterpret_cast<const f32x4*>(K + krow * kDim + c4 * 4);
    const f32x4 vv = *reinterpret_cast<const f32x4*>(V + krow * kDim + c4 * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      kr[c4 * 4 + e] = kv[e];
      vr[c4 * 4 + e] = vv[e];
    }
  }
  const bool key_valid = !p.kmask || p.kmask[static_cast<size_t>(bi) * p.n + k * kBlk + kk] != 0;
  const bool key_global = pat.is_global(k);
  const int32_t* tbl = p.rand_idx ? p.rand_idx + static_cast<size_t>(h) * nb * p.r : nullptr;
  const float c = p.c;
  float dk[16], dv[16];
#pragma unroll
  for (int d = 0; d < 16; ++d) dk[d] = dv[d] = 0.f;

  for (int j0 = 0; j0 < nb; j0 += kListChunk) {
    __syncthreads();  // the previous chunk's list is no longer read
    if (threadIdx.x < 64) {
      // query blocks j0 .. j0+63 that attend k, in ascending order
      const int j = j0 + threadIdx.x;
      bool att = false;
      if (j < nb) {
        att = key_global || pat.is_global(j) || pat.in_window(j, k);
        if (!att && tbl)
          for (int t = 0; t < p.r; ++t) att |= tbl[static_cast<size_t>(j) * p.r + t] == k;
      }
      const uint64_t m = __ballot(att);
      if (att) jlist[mask_rank(m)] = j;
      if (threadIdx.x == 0) jcount = static_cast<int>(__popcll(m));
    }
    __syncthreads();
    const int cnt = jcount;
    for (int u = 0; u < cnt; ++u) {
      const int j = jlist[u];
      __syncthreads();  // tiles and products of the previous query block are no longer read
      const size_t jrow0 = bh_row0 + static_cast<size_t>(j) * kBlk;
      load_tile_f32(Q + jrow0 * kDim, lds_q);
      load_tile_f32(dO + jrow0 * kDim, lds_do);
      if (threadIdx.x < 64) {
        lds_lse[threadIdx.x] = p.Lvec[jrow0 + threadIdx.x];
        lds_d[threadIdx.x] = p.Dvec[jrow0 + threadIdx.x];
      }
      __syncthreads();
      for (int t = 0; t < 16; ++t) {
        const int i = part * 16 + t;
        const float s = dot_row(kr, lds_q + i * kTileStride);
        const float dp = dot_row(vr, lds_do + i * kTileStride);
        const float pr = key_valid ? fast_exp2(__builtin_fmaf(s, c, -lds_lse[i])) : 0.f;
        // attention dropout: dV takes the kept, rescaled probabilities; dP is masked the same way
        float mr = 1.f;
        if (p.drop.thr)
          mr = drop_keep(p.drop, static_cast<uint32_t>(jrow0 + i), static_cast<uint32_t>(k * kBlk + kk))
                   ? p.drop.rs : 0.f;
        lds_p[i * (kBlk + 1) + kk] = pr * mr;
        lds_ds[i * (kBlk + 1) + kk] = pr * (dp * mr - lds_d[i]);
      }
      __syncthreads();
      for (int i = 0; i < kBlk; ++i) {
        const float pr = lds_p[i * (kBlk + 1) + kk];
        const float ds = lds_ds[i * (kBlk + 1) + kk];
        const float* qrow = lds_q + i * kTileStride + part * 16;
        const float* grow = lds_do + i * kTileStride + part * 16;
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
          const f32x4 qv = *reinterpret_cast<const f32x4*>(qrow + c4 * 4);
          const f32x4 gv = *reinterpret_cast<const f32x4*>(grow + c4 * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            dk[c4 * 4 + e] = __builtin_fmaf(ds, qv[e], dk[c4 * 4 + e]);
            dv[c4 * 4 + e] = __builtin_fmaf(pr, gv[e], dv[c4 * 4 + e]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int c4 = 0; c4 < 4; ++c4) {
    f32x4 a, b;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      a[e] = dk[c4 * 4 + e] * p.scale;
      b[e] = dv[c4 * 4 + e];
    }
    *reinterpret_cast<f32x4*>(p.dK + krow * kDim + part * 16 + c4 * 4) = a;
    *reinterpret_cast<f32x4*>(p.dV + krow * kDim + part * 16 + c4 * 4) = b;
  }
}

int launch_bwd_f32(const BwdParams& p, hipStream_t stream) {
  const unsigned grid = static_cast<unsigned>(p.BH) * p.nb;
  if (grid == 0) return BB_OK;
  hipLaunchKernelGGL(bwd_f32_dq_kernel, dim3(grid), dim3(kF32Threads), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) {
    hipLaunchKernelGGL(bwd_f32_dkv_kernel, dim3(grid), dim3(kF32Threads), 0, stream, p);
    e = hipGetLastError();
  }
  if (e != hipSuccess) {
    fprintf(stderr, "bigbird: launch of the fp32 backward kernels failed: %s\n", hipGetErrorString(e));
    return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
