// bf16 forward kernel: the tuned path of the BERT-shaped workloads.
//
// Same mathematics as the fp32 kernel (eq. (AT) per head on the App. D pattern),
// with the machinery the bf16 MFMA rate asks for:
//   * K and V tiles go global -> LDS directly (no registers in between), two
//     buffers each, one workgroup barrier per key block;
//   * the scores of key block i+1 are issued to the MFMA pipe before the softmax
//     of block i runs on the vector ALU, so the two pipes overlap inside a wave;
//   * V^T operands come from the transposing LDS read;
//   * the softmax reference exponent moves only when a row maximum grows by more
//     than 2^8, so the accumulator rescale is rare; row sums are taken from the
//     bf16-rounded probabilities with the packed dot instruction.
#include "fwd_epilogue.h"
#include "tile_ops.h"

#include <cstdio>
#include <type_traits>

namespace bb {

namespace {

constexpr float kLazyLog2 = 8.f;  // rescale when a row maximum grows by more than 2^8

__device__ __forceinline__ void zero_acc(f32x16 (&a)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) a[t][r] = 0.f;
}

}  // namespace

#ifndef BB_FWD_WAVES_PER_EU
#define BB_FWD_WAVES_PER_EU 2
#endif

// Schedule of one work item (key blocks k_0 .. k_{cnt-1}); K and V each have two
// LDS buffers:
//   prologue   load K0 -> Kbuf0, V0 -> Vbuf0, K1 -> Kbuf1;  S(0) = K0 Q^T
//   step i     wait for K(i+1), V(i); barrier            (one barrier per key block)
//              load K(i+2) -> Kbuf[i&1], V(i+1) -> Vbuf[(i+1)&1]   (a full step of slack)
//              issue S(i+1) = K(i+1) Q^T on the MFMA pipe ...
//              ... while the VALU does the softmax of S(i)
//              O += V(i)^T P(i)^T, its MFMAs interleaved with the exponentials
// so within one wave the matrix pipe works on the next block's scores while the
// vector pipe exponentiates the current block's.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(BB_FWD_WAVES_PER_EU)))
void fwd_kernel_bf16(FwdParams p) {
  constexpr int kTile = kBlk * kDim * 2;  // 8 KB
  __shared__ __attribute__((aligned(1024))) char lds_k[2 * kTile];
  __shared__ __attribute__((aligned(1024))) char lds_v[2 * kTile];
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
  const int kl = klist[lane & (kChunk - 1)];  // lane t holds list entry t & 7
  auto key_block = [&](int i) { return __builtin_amdgcn_readlane(kl, i); };

  const size_t bh_row0 = static_cast<size_t>(it.bh) * p.n;
  const size_t qrow = bh_row0 + it.j * kBlk + wv * 32 + col;
  const char* kbase = static_cast<const char*>(p.K) + bh_row0 * (kDim * 2);
  const char* vbase = static_cast<const char*>(p.V) + bh_row0 * (kDim * 2);

  // per-lane pieces of the tile loads (see tile_load_async)
  const unsigned voff = tile_load_lane_offset(wv, lane);
  const unsigned lds_k_wave = __builtin_amdgcn_readfirstlane(lds_addr(lds_k) + wv * 1024);
  const unsigned lds_v_wave = __builtin_amdgcn_readfirstlane(lds_addr(lds_v) + wv * 1024);
  auto tile_off = [&](int i) { return static_cast<size_t>(key_block(i)) * kTile; };

  if (cnt > 0) {
    tile_load_async(kbase + tile_off(0), lds_k_wave, voff);
    tile_load_async(vbase + tile_off(0), lds_v_wave, voff);
    if (cnt > 1) tile_load_async(kbase + tile_off(1), lds_k_wave + kTile, voff);
  }

  // Q^T operand (B of S^T = K Q^T): lane holds query `col`, d = 16*ks + 8*hf .. +8
  bf16x8 qb[4];
  {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.Q) + qrow * kDim);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qb[ks] = qp[ks * 2 + hf];
  }
  // Make the compiler account for the Q loads here, once, instead of at the first
  // use inside the loop (where its conservative wait would drain the tile loads).
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qb[ks]));

  f32x16 o[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_ref = neg_inf();  // reference exponent in raw score units (both halves agree)
  float l_run = 0.f;        // this lane's share of sum 2^((s - m_ref) c)
  const float c = p.c;
  const float tau = kLazyLog2 / c;

  const StraightOffsets so(lane);
  const TransposedOffsets to(lane);

  f32x16 sc[2][2];  // scores of the current and of the next key block
  if (cnt > 0) {
    // K0 landed (V0 and, if there is one, K1 may still be in flight)
    if (cnt > 1)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(4));
    BB_BARRIER();
    bf16x8 ka[2][4];
    so.read(lds_k, ka);
    zero_acc(sc[0]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        sc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t][ks], qb[ks], sc[0][t], 0, 0, 0);
  }

  // One key block.  P = parity of i (which buffers), MORE = a block i+1 exists.
  // The instruction stream is laid out so that about one MFMA is issued per ten
  // vector instructions: the eight MFMAs of the next block's scores and the eight of
  // this block's value product are spread over the row-maximum and the four
  // exponential groups (the vector ALU is the longer pipe at d = 64).
  auto step = [&](auto parity, auto more_tag, int i) {
    constexpr int P = decltype(parity)::value;
    constexpr bool MORE = decltype(more_tag)::value;
    f32x16(&s)[2] = sc[P];
    f32x16(&sn)[2] = sc[P ^ 1];
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, key_block(i));

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // K(i+1) and V(i) have landed
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);     // and this wave's reads of the buffers reused below are done
    BB_BARRIER();
    if constexpr (MORE) {
      if (i + 2 < cnt) tile_load_async(kbase + tile_off(i + 2), lds_k_wave + P * kTile, voff);
      tile_load_async(vbase + tile_off(i + 1), lds_v_wave + (P ^ 1) * kTile, voff);
    }
    // all LDS operand reads of this step, up front: K(i+1) for the next scores, V(i)^T for
    // this block's value product (see TransposedOffsets for the key order)
    bf16x8 ka[2][4], va[2][4];
    if constexpr (MORE) {
      so.read(lds_k + (P ^ 1) * kTile, ka);
      zero_acc(sn);
    }
    to.read(lds_v + P * kTile, va);
    auto next_scores = [&](int idx) {  // MFMA idx (0..7) of S(i+1) = K(i+1) Q^T
      if constexpr (MORE) {
        const int ks = idx >> 1, t = idx & 1;
        sn[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t][ks], qb[ks], sn[t], 0, 0, 0);
      }
    };

    if (vbits != ~0ull) {  // partly padded block: masked keys get -inf
      const uint64_t mine = vbits >> (hf * 4);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!((mine >> (t * 32 + acc_row(r, 0))) & 1)) s[t][r] = neg_inf();
    }

    // ---- row maximum (base-2 online softmax with a lazily moved reference)
    next_scores(0);
    next_scores(1);
    float mloc = neg_inf();
#pragma unroll
    for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[0][r]);
    next_scores(2);
#pragma unroll
    for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[1][r]);
    next_scores(3);
    mloc = half_max(mloc);
    __builtin_amdgcn_sched_barrier(0);
    if (__any(mloc > m_ref + tau)) {
      const float m_new = fmaxf(m_ref, mloc);
      const float m_use = (m_new == neg_inf()) ? 0.f : m_new;
      const float alpha = fast_exp2((m_ref - m_use) * c);
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
      m_ref = m_new;
    }
    const float mc = (m_ref == neg_inf()) ? 0.f : m_ref * c;

    // ---- four groups of 16 keys: exponentials, then the group's share of O^T += V^T P^T
    const bf16x2 ones = {static_cast<__bf16>(1.f), static_cast<__bf16>(1.f)};
#pragma unroll
    for (int sg = 0; sg < 4; ++sg) {
      bf16x8 pb;
#pragma unroll
      for (int kk = 0; kk < 8; kk += 2) {
        const int t = sg >> 1, r = (sg & 1) * 8 + kk;
        const float p0 = fast_exp2(__builtin_fmaf(s[t][r], c, -mc));
        const float p1 = fast_exp2(__builtin_fmaf(s[t][r + 1], c, -mc));
        const bf16x2 pk = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
        pb[kk] = pk[0];
        pb[kk + 1] = pk[1];
        l_run = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l_run, false);
        if (sg < 2 && kk == 2) next_scores(4 + 2 * sg);
        if (sg < 2 && kk == 6) next_scores(5 + 2 * sg);
      }
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt][sg], pb, o[dt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  {
    using T = std::true_type;
    using F = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    int i = 0;
    for (; i + 2 < cnt; i += 2) {
      step(P0{}, T{}, i);
      step(P1{}, T{}, i + 1);
    }
    if (cnt - i == 2) {
      step(P0{}, T{}, i);
      step(P1{}, F{}, i + 1);
    } else if (cnt - i == 1) {
      step(P0{}, F{}, i);
    }
  }

  const float l_tot = half_sum(l_run);
  fwd_store<true>(p, it, o, m_ref, l_tot, c, qrow, wv * 32 + col, hf);
}

int launch_fwd_bf16_main(const FwdParams& p, unsigned grid, hipStream_t stream) {
  hipLaunchKernelGGL(fwd_kernel_bf16, dim3(grid), dim3(kThreads), 0, stream, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    fprintf(stderr, "bigbird: launch of fwd_kernel_bf16 failed: %s\n", hipGetErrorString(e));
    return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
