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
  const unsigned voff = ((wv * 8 + (lane >> 3)) * 128) + ((((lane & 7) ^ (lane >> 3))) << 4);
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

  // LDS byte offsets of this lane's operand pieces (fixed for the whole item)
  int koff[2][4];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[t][ks] = tile_off_bf16(t * 32 + col, ks * 2 + hf);
  const int gq = lane >> 4, li = lane & 15;
  int voff_tr[2];  // V^T operand: row (4*hf + li/4) of a 16-key group, 8-byte piece of a d chunk
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
    voff_tr[dt] = tile_off_bf16(hf * 4 + (li >> 2), dt * 4 + (gq & 1) * 2 + ((li & 3) >> 1)) + (li & 1) * 8;

  // S^T = K Q^T for the tile in K buffer `buf`: rows = 64 keys (two MFMA tiles), columns =
  // this wave's 32 queries.
  auto scores = [&](int buf, f32x16 (&s)[2]) {
    const char* kt = lds_k + buf * kTile;
    bf16x8 ka[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) ka[t][ks] = *reinterpret_cast<const bf16x8*>(kt + koff[t][ks]);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t][ks], qb[ks], s[t], 0, 0, 0);
  };

  f32x16 sc[2][2];  // scores of the current and of the next key block
  if (cnt > 0) {
    // K0 landed (V0 and, if there is one, K1 may still be in flight)
    if (cnt > 1)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(4));
    BB_BARRIER();
    scores(0, sc[0]);
  }

  auto step = [&](auto parity, int i) {
    constexpr int P = decltype(parity)::value;
    f32x16(&s)[2] = sc[P];
    const int kb = key_block(i);
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, kb);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // K(i+1) and V(i) have landed
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);     // and this wave's reads of the buffers reused below are done
    BB_BARRIER();
    if (i + 2 < cnt) tile_load_async(kbase + tile_off(i + 2), lds_k_wave + P * kTile, voff);
    if (i + 1 < cnt) {
      tile_load_async(vbase + tile_off(i + 1), lds_v_wave + (P ^ 1) * kTile, voff);
      scores(P ^ 1, sc[P ^ 1]);  // next block's scores: runs on the MFMA pipe under the softmax below
    }

    if (vbits != ~0ull) {  // partly padded block: masked keys get -inf
      const uint64_t mine = vbits >> (hf * 4);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!((mine >> (t * 32 + acc_row(r, 0))) & 1)) s[t][r] = neg_inf();
    }

    // ---- online softmax, base 2, lazily moved reference
    float mloc = neg_inf();
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[t][r]);
    mloc = half_max(mloc);
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

    // V^T operand (A of O^T += V^T P^T): lane holds d = 32*dt + col and, in MFMA
    // contraction slot 8*hf + kk, the key 16*sg + 4*hf + kk (kk < 4) or + 8 + kk - 4.
    const char* vt = lds_v + P * kTile;
    bf16x8 va[2][4];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) {
        // rows 16*sg + {0, 8} + (4*hf + li/4): a multiple of 8 added to the row keeps the swizzle
        const s16x4 lo = lds_read_tr16(vt + voff_tr[dt] + sg * 2048);
        const s16x4 hi = lds_read_tr16(vt + voff_tr[dt] + sg * 2048 + 1024);
        union { struct { s16x4 a, b; } h2; bf16x8 v; } u;
        u.h2.a = lo;
        u.h2.b = hi;
        va[dt][sg] = u.v;
      }
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
      }
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt][sg], pb, o[dt], 0, 0, 0);
    }
  };

  for (int i = 0; i < cnt; i += 2) {
    step(std::integral_constant<int, 0>{}, i);
    if (i + 1 < cnt) step(std::integral_constant<int, 1>{}, i + 1);
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
