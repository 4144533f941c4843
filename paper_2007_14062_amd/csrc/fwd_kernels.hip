// Forward kernels: the fp32 fused kernel (S^T = K Q^T -> online softmax ->
// O^T += V^T P^T per query block and slice of its key-block list), the merge of
// sliced rows, and the launch logic.  The bf16 fused kernel is in fwd_bf16.hip.
//
// Eq. (AT) of Sec. 2 per head on the blocked pattern of App. D.  Each block pair
// is a dense 64x64x64 contraction, which is what the MFMA units are for.  The
// scores are produced transposed (keys along MFMA rows, queries along MFMA
// columns) so that one lane owns one query column: the row maximum and row sum of
// the softmax are in-lane reductions plus one exchange between the two 32-lane
// halves, and the probabilities sit in registers exactly where the second MFMA
// wants its B operand (the contraction order over keys is free, so V^T is read
// from LDS in the matching permuted key order).
#include "fwd_epilogue.h"

#include <cstdio>

namespace bb {

namespace {

constexpr int kTileBytesF32 = kBlk * kF32Stride * 4;            // 17 KB, rows padded to 68 floats
constexpr int kVecPerThreadF32 = kBlk * kDim * 4 / 16 / kThreads;  // 8 x 16 bytes per thread

// Global -> registers: one 64x64 fp32 tile of K or V, 16 bytes per lane per step, coalesced.
__device__ __forceinline__ void tile_fetch_f32(const float* base, size_t row0, u32x4* regs) {
  const int tid = threadIdx.x;
  const char* p = reinterpret_cast<const char*>(base + row0 * kDim);
#pragma unroll
  for (int i = 0; i < kVecPerThreadF32; ++i) {
    const int idx = i * kThreads + tid;
    regs[i] = *reinterpret_cast<const u32x4*>(p + (idx >> 4) * 256 + (idx & 15) * 16);
  }
}

// Registers -> LDS, rows padded so that the column reads of the MFMA operands spread over banks.
__device__ __forceinline__ void tile_store_f32(char* lds, const u32x4* regs) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < kVecPerThreadF32; ++i) {
    const int idx = i * kThreads + tid;
    *reinterpret_cast<u32x4*>(lds + ((idx >> 4) * kF32Stride + (idx & 15) * 4) * 4) = regs[i];
  }
}

}  // namespace

// fp32 end to end (the small correctness workload): fp32 MFMA 32x32x2, tiles staged
// through registers into one LDS buffer each, plain online softmax.
__global__ __launch_bounds__(kThreads) void fwd_kernel_f32(FwdParams p) {
  __shared__ __attribute__((aligned(16))) char lds_k[kTileBytesF32];
  __shared__ __attribute__((aligned(16))) char lds_v[kTileBytesF32];
  __shared__ int klist[kChunkMax];

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  WorkItem it;
  if (!decode_item(p.split, pat, p.BH, blockIdx.x, &it)) return;
  const int bi = it.bh / p.H, h = it.bh % p.H;
  const int lane = lane_id(), wv = threadIdx.x >> 6;
  const int hf = lane >> 5, col = lane & 31;

  // (a query block without a valid position, if the caller asked for those to be skipped, is an
  // empty row: O = 0, LSE = -inf through the usual end of an item)
  const bool skip = p.skip_q && key_valid_bits(p.kmask, bi, p.n, it.j) == 0;
  const int cnt = skip ? 0 : build_key_list(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, it.j, it.row_global,
                                            it.chunk, klist);
  __syncthreads();

  const size_t bh_row0 = static_cast<size_t>(it.bh) * p.n;    // first row of this (batch, head)
  const size_t qrow = bh_row0 + it.j * kBlk + wv * 32 + col;  // this lane's query row
  const float* Kp = static_cast<const float*>(p.K);
  const float* Vp = static_cast<const float*>(p.V);

  // Q^T operand: MFMA contraction slot hf of step (u, e) is d = 8u + 4hf + e.
  f32x4 qf[8];
  {
    const f32x4* qp = reinterpret_cast<const f32x4*>(static_cast<const float*>(p.Q) + qrow * kDim);
#pragma unroll
    for (int u = 0; u < 8; ++u) qf[u] = qp[u * 2 + hf];
  }

  f32x16 o[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  // attention dropout: the key of this lane's row of the keep mask
  const uint32_t drop_rk = p.drop.thr ? drop_row_key(p.drop, static_cast<uint32_t>(qrow)) : 0u;
  float m_run = neg_inf();  // running maximum of the raw scores q.k (both halves agree)
  float l_run = 0.f;        // this lane's share of the running sum of 2^((q.k - m) c)
  const float c = p.c;

  u32x4 kreg[kVecPerThreadF32], vreg[kVecPerThreadF32];
  if (cnt > 0) {
    const size_t krow0 = bh_row0 + static_cast<size_t>(klist[0]) * kBlk;
    tile_fetch_f32(Kp, krow0, kreg);
    tile_fetch_f32(Vp, krow0, vreg);
  }

  for (int i = 0; i < cnt; ++i) {
    const int kb = klist[i];
    __syncthreads();  // everyone is done reading the previous tiles
    tile_store_f32(lds_k, kreg);
    tile_store_f32(lds_v, vreg);
    __syncthreads();
    if (i + 1 < cnt) {
      const size_t krow0 = bh_row0 + static_cast<size_t>(klist[i + 1]) * kBlk;
      tile_fetch_f32(Kp, krow0, kreg);
      tile_fetch_f32(Vp, krow0, vreg);
    }
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, kb);

    // ---- S^T tile: rows = 64 keys (two 32-row MFMA tiles), columns = this wave's 32 queries
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
      const float* kr = reinterpret_cast<const float*>(lds_k) + (t * 32 + col) * kF32Stride + hf * 4;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(kr + u * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          s[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], qf[u][e], s[t], 0, 0, 0);
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

    // ---- attention dropout: the row sums above are those of the undropped probabilities; what
    // multiplies V is the kept part (registers r, r+1 are keys 2m, 2m+1: one word of the mask)
    if (p.drop.thr) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const uint32_t key = static_cast<uint32_t>(kb * kBlk + t * 32 + acc_row(r, hf));
          const uint32_t wd = drop_word(drop_rk, key >> 1);
          if (!drop_keep_even(wd, p.drop.thr)) s[t][r] = 0.f;
          if (!drop_keep_odd(wd, p.drop.thr)) s[t][r + 1] = 0.f;
        }
    }

    // ---- O^T += V^T P^T: the S^T accumulator is the B operand as it stands; slot hf of
    // register r is key 32t + acc_row(r, hf), and V is read in that same key order.
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

  const float l_tot = half_sum(l_run);
  fwd_store<false>(p, it, o, m_run, l_tot, c, qrow, wv * 32 + col, hf);
}

// Merge the slices of a split row: M = max m_c, L = sum l_c 2^(m_c - M),
// O = sum O~_c 2^(m_c - M) / L, LSE = (M + log2 L) ln 2.  Four workgroups per
// (batch, head, split row), 16 queries each; thread t owns 4 d columns of query
// t/16, so a wavefront reads four full 256-byte rows of every partial.
constexpr int kCombineThreads = 256;
constexpr int kCombineSplit = 4;  // workgroups per 64-query block

template <bool BF16>
__global__ __launch_bounds__(kCombineThreads) void fwd_combine_kernel(FwdParams p) {
  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const int rows_per_bh = p.cmb_g_rows + p.cmb_s_rows;
  const int part = blockIdx.x % kCombineSplit;
  const int rowid = blockIdx.x / kCombineSplit;
  const int bh = rowid / rows_per_bh, rr = rowid % rows_per_bh;
  int j, nchunks, slot0;
  if (rr < p.cmb_g_rows) {
    j = pat.global_block(rr);
    nchunks = p.cmb_g_n;
    slot0 = bh * p.slots_per_bh + rr * p.cmb_g_n;
  } else {
    const int t = rr - p.cmb_g_rows;
    j = pat.sparse_block(t);
    nchunks = p.cmb_s_n;
    slot0 = bh * p.slots_per_bh + p.cmb_g_rows * p.cmb_g_n + t * p.cmb_s_n;
  }
  const int q = part * 16 + (threadIdx.x >> 4), d0 = (threadIdx.x & 15) * 4;
  const float* ml = p.part_ml + static_cast<size_t>(slot0) * (2 * kBlk) + q;
  const float* po = p.part_o + static_cast<size_t>(slot0) * (kBlk * kDim) + q * kDim + d0;
  float M = neg_inf();
  for (int cidx = 0; cidx < nchunks; ++cidx) M = fmaxf(M, ml[cidx * (2 * kBlk)]);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float L = 0.f;
  if (M != neg_inf()) {
    constexpr int U = 8;  // partials in flight per thread
    for (int c0 = 0; c0 < nchunks; c0 += U) {
      f32x4 v[U];
      float wgt[U], lc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int cidx = c0 + u < nchunks ? c0 + u : nchunks - 1;
        v[u] = *reinterpret_cast<const f32x4*>(po + static_cast<size_t>(cidx) * (kBlk * kDim));
        const float mcur = ml[cidx * (2 * kBlk)];
        lc[u] = ml[cidx * (2 * kBlk) + kBlk];
        wgt[u] = (c0 + u < nchunks && mcur != neg_inf()) ? fast_exp2(mcur - M) : 0.f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        L += lc[u] * wgt[u];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += v[u][e] * wgt[u];
      }
    }
  }
  const float inv = L > 0.f ? p.drop.rs / L : 0.f;  // (rs: 1, or the dropout scale)
  const size_t row = static_cast<size_t>(bh) * p.n + j * kBlk + q;
  if ((threadIdx.x & 15) == 0) p.LSE[row] = L > 0.f ? (M + fast_log2(L)) * kLn2 : neg_inf();
  if constexpr (BF16) {
    bf16x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(acc[e] * inv);
    *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.O) + row * kDim + d0) = v;
  } else {
    f32x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = acc[e] * inv;
    *reinterpret_cast<f32x4*>(static_cast<float*>(p.O) + row * kDim + d0) = v;
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
  if (bf16) {
    const int st = launch_fwd_bf16_main(p, stream);
    if (st != BB_OK) return st;
  } else {
    const RowSplit& s = p.split;
    const unsigned grid = static_cast<unsigned>(kXcd) * s.bh_rounds * s.items_per_bh;
    if (grid == 0) return BB_OK;
    hipLaunchKernelGGL(fwd_kernel_f32, dim3(grid), dim3(kThreads), 0, stream, p);
    if (launch_failed("fwd_kernel_f32")) return BB_ERR_LAUNCH;
  }
  const int rows_per_bh = p.cmb_g_rows + p.cmb_s_rows;
  if (rows_per_bh > 0) {
    const unsigned cgrid = static_cast<unsigned>(p.BH) * rows_per_bh * kCombineSplit;
    if (bf16)
      hipLaunchKernelGGL(fwd_combine_kernel<true>, dim3(cgrid), dim3(kCombineThreads), 0, stream, p);
    else
      hipLaunchKernelGGL(fwd_combine_kernel<false>, dim3(cgrid), dim3(kCombineThreads), 0, stream, p);
    if (launch_failed("fwd_combine_kernel")) return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
