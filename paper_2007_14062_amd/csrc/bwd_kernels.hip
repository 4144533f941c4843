// Backward kernels (bf16 storage, fp32 gradients).  The paper gives no backward
// pass; this is the calculus of eq. (AT) of Sec. 2 on the blocked pattern of App. D.
// With P the row softmax recomputed from Q, K and the forward's LSE:
//   dV = P^T dO;  dP = dO V^T;  D_i = sum_c dO_ic O_ic;  dS = P o (dP - D);
//   dQ = scale dS K;  dK = scale dS^T Q.
//
// Two gather kernels, no atomics:
//   * bwd_dq_kernel walks the key-block list of a query block (the forward's
//     decomposition): S^T, dP^T and dS^T are [keys x queries] tiles, one lane per
//     query, and dQ^T += K^T dS^T.  It also computes the row sums D (and leaves them
//     in the workspace for the second kernel).
//   * bwd_dkv_kernel walks the query-block list of a key block -- the inverse of the
//     pattern: the global query blocks, the window, and the rows of rand_idx that
//     name this key block (found by scanning the head's table) -- with S, dP, dS as
//     [queries x keys] tiles, one lane per key, dV^T += dO^T P and dK^T += Q^T dS.
// Rows / columns of global blocks are cut into slices of 8 blocks whose partial sums
// are added in slice order by bwd_reduce_kernel (bit-reproducible).
#include "bwd_kernels.h"
#include "tile_ops.h"

#include <cstdio>

namespace bb {

namespace {

constexpr int kTile = kBlk * kDim * 2;  // one 64x64 bf16 tile: 8 KB

__device__ __forceinline__ void zero_acc(f32x16 (&a)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) a[t][r] = 0.f;
}

// Stores a [64 x 32] accumulator pair whose rows are d and whose column is this lane's
// sequence position `row` (a query for dQ, a key for dK/dV): dst[row][d0 .. d0+3].
__device__ __forceinline__ void store_acc_rows(float* dst_row, const f32x16 (&a)[2], int hf) {
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = a[dt][r4 * 4 + e];
      *reinterpret_cast<f32x4*>(dst_row + dt * 32 + acc_row(r4 * 4, hf)) = v;
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------
// dQ: one work item = (batch*head, query block j, slice of <= 8 key blocks of j's list)
// ---------------------------------------------------------------------------------------
// kDrop: attention dropout, dP = M / (1 - p) o (dO V^T) with M the keep mask (a second instance of
// the kernel, so that the one without dropout keeps its registers and its schedule).
template <bool kDrop>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2)))
void bwd_dq_kernel(BwdParams p) {
  __shared__ __attribute__((aligned(1024))) char lds_k[2 * kTile];
  __shared__ __attribute__((aligned(1024))) char lds_v[2 * kTile];
  // The key list lives in the second V buffer, which is not written before the first barrier of
  // the loop; by then every lane holds its entry in a register.
  int* const klist = reinterpret_cast<int*>(lds_v + kTile);

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  WorkItem it;
  if (!decode_item(p.split, pat, p.BH, blockIdx.x, &it)) return;
  const int bi = it.bh / p.H, h = it.bh % p.H;
  const int lane = lane_id(), wv = threadIdx.x >> 6;
  const int hf = lane >> 5, col = lane & 31;

  // a query block that the forward did not compute (no valid position, and the caller asked for
  // such blocks to be skipped): no key block, D = 0, probabilities 0
  const bool skip = p.skip_q && key_valid_bits(p.kmask, bi, p.n, it.j) == 0;
  const int cnt = skip ? 0 : build_key_list(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, it.j, it.row_global,
                                            it.chunk, klist);
  __syncthreads();
  const int kl = klist[lane & (kChunkMax - 1)];
  auto key_block = [&](int i) { return __builtin_amdgcn_readlane(kl, i); };

  const size_t bh_row0 = static_cast<size_t>(it.bh) * p.n;
  const size_t qrow = bh_row0 + it.j * kBlk + wv * 32 + col;
  const char* kbase = static_cast<const char*>(p.K) + bh_row0 * (kDim * 2);
  const char* vbase = static_cast<const char*>(p.V) + bh_row0 * (kDim * 2);
  const unsigned voff = tile_load_lane_offset(wv, lane);
  const unsigned lds_k_wave = __builtin_amdgcn_readfirstlane(lds_addr(lds_k) + wv * 1024);
  const unsigned lds_v_wave = __builtin_amdgcn_readfirstlane(lds_addr(lds_v) + wv * 1024);
  auto tile_off = [&](int i) { return static_cast<size_t>(key_block(i)) * kTile; };

  if (cnt > 0) {
    tile_load_async(kbase + tile_off(0), lds_k_wave, voff);
    tile_load_async(vbase + tile_off(0), lds_v_wave, voff);
  }

  // B operands kept for the whole item: Q^T and dO^T, lane = query `col`, d = 16ks + 8hf .. +8
  bf16x8 qb[4], dob[4];
  {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.Q) + qrow * kDim);
    const bf16x8* dp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.dO) + qrow * kDim);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qb[ks] = qp[ks * 2 + hf];
      dob[ks] = dp[ks * 2 + hf];
    }
  }
  // D_i = sum_c dO_ic O_ic and LSE_i log2(e) of this lane's query (+inf where the forward found
  // no valid key, so that the recomputed probabilities of such a row are 0).  The lane pair
  // (l, l+32) shares a query and holds complementary halves of its d range.  The first slice of
  // a row also leaves both values in the workspace for the dK/dV kernel, which runs after this one.
  float dsum, lse2;
  {
    const bf16x8* op = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.O) + qrow * kDim);
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 ob = op[ks * 2 + hf];
#pragma unroll
      for (int e = 0; e < 8; ++e) part += static_cast<float>(dob[ks][e]) * static_cast<float>(ob[e]);
    }
    dsum = skip ? 0.f : half_sum(part);
    const float lse = p.LSE[qrow];
    lse2 = (skip || lse == neg_inf()) ? __builtin_inff() : lse * kLog2e;
    if (it.chunk == 0 && hf == 0) {
      p.Dvec[qrow] = -dsum;  // negated: the other kernel starts its dP accumulators from it
      p.Lvec[qrow] = lse2;
    }
  }
  // let the compiler settle these loads here, not inside the loop (see the forward kernel)
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qb[ks]), "+v"(dob[ks]));
  asm volatile("" : "+v"(lse2), "+v"(dsum));

  const StraightOffsets so(lane);
  const TransposedOffsets to(lane);
  f32x16 dq[2];
  zero_acc(dq);
  const float c = p.c;
  f32x16 neg_d;
#pragma unroll
  for (int r = 0; r < 16; ++r) neg_d[r] = kDrop ? 0.f : -dsum;  // (with dropout D is subtracted after the mask)
  uint32_t drop_rk = 0u;
  if constexpr (kDrop) drop_rk = drop_row_key(p.drop, static_cast<uint32_t>(qrow));

  for (int i = 0; i < cnt; ++i) {
    const int buf = i & 1;
    const int kb = key_block(i);
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, kb);

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // K(i), V(i) landed
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);     // our reads of the other buffers are done
    BB_BARRIER();
    if (i + 1 < cnt) {
      tile_load_async(kbase + tile_off(i + 1), lds_k_wave + (buf ^ 1) * kTile, voff);
      tile_load_async(vbase + tile_off(i + 1), lds_v_wave + (buf ^ 1) * kTile, voff);
    }
    const char* kt = lds_k + buf * kTile;
    const char* vt = lds_v + buf * kTile;

    // S^T = K Q^T and dP^T = V dO^T: rows = 64 keys, columns = this wave's 32 queries
    // (dP^T starts from -D: every element of a lane's accumulators belongs to the lane's query,
    // so the subtraction in dS = P o (dP - D) costs no vector instruction)
    f32x16 s[2], dp[2];
    zero_acc(s);
    dp[0] = neg_d;
    dp[1] = neg_d;
    bf16x8 ka[2][4], va[2][4];
    so.read(kt, ka);
    so.read(vt, va);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t][ks], qb[ks], s[t], 0, 0, 0);
    if (vbits != ~0ull) {  // partly padded block: masked keys get probability 0
      const uint64_t mine = vbits >> (hf * 4);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!((mine >> (t * 32 + acc_row(r, 0))) & 1)) s[t][r] = neg_inf();
    }
    // P^T = 2^(S^T c - LSE log2e) on the vector ALU while the matrix pipe computes dP^T (the issue
    // order "one MFMA, eight vector instructions" is pinned: left alone the compiler queues the
    // MFMAs first, and the wave can issue nothing else meanwhile)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        dp[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[t][ks], dob[ks], dp[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[t][r] = fast_exp2(__builtin_fmaf(s[t][r], c, -lse2));
        asm volatile("" : "+v"(s[t][r]));  // computed here, beside the MFMAs, not where it is used
      }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 8, 0);
    }
    if constexpr (kDrop) {
      // registers r, r + 1 are keys 2m, 2m + 1: one word of the mask
      const float rs = p.drop.rs, nd = -dsum;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const uint32_t key = static_cast<uint32_t>(kb * kBlk + t * 32 + acc_row(r, hf));
          const uint32_t wd = drop_word(drop_rk, key >> 1);
          dp[t][r] = drop_keep_even(wd, p.drop.thr) ? __builtin_fmaf(dp[t][r], rs, nd) : nd;
          dp[t][r + 1] = drop_keep_odd(wd, p.drop.thr) ? __builtin_fmaf(dp[t][r + 1], rs, nd) : nd;
        }
    }
    // dS^T = P^T o (dP^T - D)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] *= dp[t][r];
    bf16x8 dsb[4];
    pack_acc_bf16(s, dsb);

    // dQ^T += K^T dS^T: rows = d, columns = queries, contraction over the 64 keys
    bf16x8 kta[2][4];
    to.read(kt, kta);
#pragma unroll
    for (int sg = 0; sg < 4; ++sg)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kta[dt][sg], dsb[sg], dq[dt], 0, 0, 0);
  }

#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] *= p.scale;
  if (it.nchunks == 1) {
    store_acc_rows(p.dQ + qrow * kDim, dq, hf);
  } else {
    float* po = p.part_dq + static_cast<size_t>(it.slot) * (kBlk * kDim);
    store_acc_rows(po + (wv * 32 + col) * kDim, dq, hf);
  }
}

// ---------------------------------------------------------------------------------------
// dK, dV: one work item = (batch*head, key block k[, slice of its query-block list])
// ---------------------------------------------------------------------------------------
// kDrop: attention dropout (see bwd_dq_kernel): dV takes the kept probabilities (rescaled at the
// end), dP is masked and rescaled before D is subtracted.  The row keys of the mask for the 64
// queries of a list entry are staged in LDS beside LSE and D.
template <bool kDrop>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2)))
void bwd_dkv_kernel(BwdParams p) {
  __shared__ __attribute__((aligned(256))) uint32_t lds_rk[kDrop ? 2 * kBlk : 4];
  __shared__ __attribute__((aligned(1024))) char lds_q[2 * kTile];
  __shared__ __attribute__((aligned(1024))) char lds_do[2 * kTile];
  __shared__ __attribute__((aligned(256))) float lds_lse[2 * kBlk];
  __shared__ __attribute__((aligned(256))) float lds_d[2 * kBlk];
  __shared__ int jlist[kMaxBwdBlocks];

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const int nb = p.nb;
  // workgroup id -> (batch*head, item); id % 8 is the die, as in the forward
  const int xcd = blockIdx.x % kXcd;
  const unsigned qidx = blockIdx.x / kXcd;
  const int bh = (qidx / p.kv_items_per_bh) * kXcd + xcd;
  if (bh >= p.BH) return;
  const int item = qidx % p.kv_items_per_bh;
  const int bi = bh / p.H, h = bh % p.H;
  const int lane = lane_id(), wv = threadIdx.x >> 6;
  const int hf = lane >> 5, col = lane & 31;

  const int nglob = p.g * p.cq;
  const bool key_global = item < nglob;
  int k, chunk = 0, slot = 0;
  if (key_global) {
    k = pat.global_block(item / p.cq);
    chunk = item % p.cq;
    slot = (bh * p.g + item / p.cq) * p.cq + chunk;
  } else {
    k = pat.sparse_block(item - nglob);
  }
  const bool split = key_global && p.cq > 1;

  const size_t bh_row0 = static_cast<size_t>(bh) * p.n;
  const size_t krow = bh_row0 + k * kBlk + wv * 32 + col;  // this lane's key
  float* dk_dst = split ? p.part_dk + static_cast<size_t>(slot) * (kBlk * kDim) + (wv * 32 + col) * kDim
                        : p.dK + krow * kDim;
  float* dv_dst = split ? p.part_dv + static_cast<size_t>(slot) * (kBlk * kDim) + (wv * 32 + col) * kDim
                        : p.dV + krow * kDim;

  f32x16 dk[2], dv[2];
  zero_acc(dk);
  zero_acc(dv);

  uint64_t vbits = ~0ull;
  if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, k);
  if (vbits == 0) {  // fully padded key block: gradients are exactly 0
    store_acc_rows(dk_dst, dk, hf);
    store_acc_rows(dv_dst, dv, hf);
    return;
  }
  const bool key_valid = (vbits >> (wv * 32 + col)) & 1;

  // ---- query blocks that attend key block k
  int cnt = 0;
  if (key_global) {
    // every query block attends a global key block (Sec. 2: A(:, i) = 1 for i in G)
    const int lo = chunk * kChunk;
    cnt = nb - lo < kChunk ? nb - lo : kChunk;
    if (cnt < 0) cnt = 0;
    if (!p.skip_q) {
      if (threadIdx.x < kChunk) jlist[threadIdx.x] = lo + threadIdx.x;
    } else {
      // without the query blocks that were not computed (both waves count, wave 0 writes)
      const bool valid = lane < cnt && block_has_valid_key(p.kmask, bi, p.n, lo + lane);
      const uint64_t m = __ballot(valid);
      if (valid && wv == 0) jlist[mask_rank(m)] = lo + lane;
      cnt = static_cast<int>(__popcll(m));
    }
  } else {
    // global query blocks, then the window, then rows of rand_idx that name k
    const int32_t* tbl = p.rand_idx ? p.rand_idx + static_cast<size_t>(h) * nb * p.r : nullptr;
    for (int c0 = 0; c0 < p.g + p.w && cnt < kMaxBwdBlocks; c0 += 64) {
      const int ci = c0 + lane;
      bool valid = false;
      int j = -1;
      if (ci < p.g) {
        j = pat.global_block(ci);
        valid = true;
      } else if (ci < p.g + p.w) {
        j = k - pat.half() + (ci - p.g);
        valid = j >= 0 && j < nb && !pat.is_global(j);
      }
      if (p.skip_q && valid) valid = block_has_valid_key(p.kmask, bi, p.n, j);
      const uint64_t m = __ballot(valid);
      const int rank = cnt + mask_rank(m);
      if (valid && rank < kMaxBwdBlocks && wv == 0) jlist[rank] = j;
      cnt += __popcll(m);
    }
    if (tbl) {
      for (int j0 = 0; j0 < nb && cnt < kMaxBwdBlocks; j0 += 64) {
        const int j = j0 + lane;
        bool valid = false;
        if (j < nb && !pat.is_global(j) && !pat.in_window(j, k)) {
          for (int t = 0; t < p.r; ++t) valid |= tbl[static_cast<size_t>(j) * p.r + t] == k;
        }
        if (p.skip_q && valid) valid = block_has_valid_key(p.kmask, bi, p.n, j);
        const uint64_t m = __ballot(valid);
        const int rank = cnt + mask_rank(m);
        if (valid && rank < kMaxBwdBlocks && wv == 0) jlist[rank] = j;
        cnt += __popcll(m);
      }
    }
    if (cnt > kMaxBwdBlocks) cnt = kMaxBwdBlocks;  // unreachable: the host bounds nb
  }
  __syncthreads();

  const char* qbase = static_cast<const char*>(p.Q) + bh_row0 * (kDim * 2);
  const char* dobase = static_cast<const char*>(p.dO) + bh_row0 * (kDim * 2);
  const float* lbase = p.Lvec + bh_row0;
  const float* dbase = p.Dvec + bh_row0;
  const unsigned voff = tile_load_lane_offset(wv, lane);
  const unsigned lds_q_wave = __builtin_amdgcn_readfirstlane(lds_addr(lds_q) + wv * 1024);
  const unsigned lds_do_wave = __builtin_amdgcn_readfirstlane(lds_addr(lds_do) + wv * 1024);
  const unsigned lds_lse_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_lse));
  const unsigned lds_d_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_d));
  // wave 0 brings LSE_j, wave 1 brings D_j (256 bytes each)
  auto stage = [&](int i, int buf) {
    const int j = __builtin_amdgcn_readfirstlane(jlist[i]);
    const size_t off = static_cast<size_t>(j) * kTile;
    tile_load_async(qbase + off, lds_q_wave + buf * kTile, voff);
    tile_load_async(dobase + off, lds_do_wave + buf * kTile, voff);
    if (wv == 0)
      vec_load_async(lbase + static_cast<size_t>(j) * kBlk, lds_lse_a + buf * (kBlk * 4), lane);
    else
      vec_load_async(dbase + static_cast<size_t>(j) * kBlk, lds_d_a + buf * (kBlk * 4), lane);
    if constexpr (kDrop) {
      if (wv == 0)
        lds_rk[buf * kBlk + lane] = drop_row_key(p.drop, static_cast<uint32_t>(bh_row0 + static_cast<size_t>(j) * kBlk + lane));
    }
  };
  if (cnt > 0) stage(0, 0);

  // B operands kept for the whole item: K^T and V^T, lane = key `col`, d = 16ks + 8hf .. +8
  bf16x8 kb[4], vb[4];
  {
    const bf16x8* kp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.K) + krow * kDim);
    const bf16x8* vp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.V) + krow * kDim);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      kb[ks] = kp[ks * 2 + hf];
      vb[ks] = vp[ks * 2 + hf];
    }
  }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(kb[ks]), "+v"(vb[ks]));

  const StraightOffsets so(lane);
  const TransposedOffsets to(lane);
  const float c = p.c;

  for (int i = 0; i < cnt; ++i) {
    const int buf = i & 1;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
    BB_BARRIER();
    if (i + 1 < cnt) stage(i + 1, buf ^ 1);
    const char* qt = lds_q + buf * kTile;
    const char* dot = lds_do + buf * kTile;

    // S = Q K^T and dP = dO V^T: rows = 64 queries of block j, columns = this wave's 32 keys
    // (dP starts from -D_q, staged with the tiles: element r of an accumulator belongs to query
    // row acc_row(r), so dS = P o (dP - D) needs no subtraction afterwards)
    const float* lq = lds_lse + buf * kBlk;
    const float* dq = lds_d + buf * kBlk;
    f32x16 s[2], dp[2];
    zero_acc(s);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dq + t * 32 + acc_row(r4 * 4, hf));
#pragma unroll
        for (int e = 0; e < 4; ++e) dp[t][r4 * 4 + e] = kDrop ? 0.f : d4[e];
      }
    {
      bf16x8 qa[2][4];
      so.read(qt, qa);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[t][ks], kb[ks], s[t], 0, 0, 0);
    }
    bf16x8 pb[4], dsb[4];
    {
      bf16x8 da[2][4];
      so.read(dot, da);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          dp[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da[t][ks], vb[ks], dp[t], 0, 0, 0);
      // P = 2^(S c - LSE_q log2e) beside the dP MFMAs; q runs along the rows.  (A padded key's
      // column is not set to 0 here: a lane's key only reaches that key's own columns of dK and
      // dV, which are cleared at the end.)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(lq + t * 32 + acc_row(r4 * 4, hf));
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            s[t][r4 * 4 + e] = fast_exp2(__builtin_fmaf(s[t][r4 * 4 + e], c, -l4[e]));
          }
        }
      if constexpr (kDrop) {
        // this lane's key against the 32 queries of its accumulator rows: the kept probabilities
        // go to dV, and dP becomes M / (1 - p) o dP - D  (the staged vector holds -D)
        const uint32_t* rkq = lds_rk + buf * kBlk;
        const uint32_t my_pair = static_cast<uint32_t>(k * kBlk + wv * 32 + col) >> 1;
        const uint32_t my_shift = (col & 1) ? 16u : 0u;
        const float rs = p.drop.rs;
        f32x16 sk[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const u32x4 k4 = *reinterpret_cast<const u32x4*>(rkq + t * 32 + acc_row(r4 * 4, hf));
            const f32x4 d4 = *reinterpret_cast<const f32x4*>(dq + t * 32 + acc_row(r4 * 4, hf));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const uint32_t wd = drop_word(k4[e], my_pair);
              const bool keep = ((wd >> my_shift) & 0x7fffu) >= p.drop.thr;
              sk[t][r4 * 4 + e] = keep ? s[t][r4 * 4 + e] : 0.f;
              dp[t][r4 * 4 + e] = keep ? __builtin_fmaf(dp[t][r4 * 4 + e], rs, d4[e]) : d4[e];
            }
          }
        pack_acc_bf16(sk, pb);
      } else {
        pack_acc_bf16(s, pb);
      }
    }

    // dV^T += dO^T P and dK^T += Q^T dS: rows = d, columns = keys, contraction over the 64 queries;
    // dS = P o (dP - D_q) and its conversion beside the dV MFMAs
    {
      bf16x8 dta[2][4];
      to.read(dot, dta);
#pragma unroll
      for (int sg = 0; sg < 4; ++sg)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dta[dt][sg], pb[sg], dv[dt], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) dp[t][r] *= s[t][r];
      pack_acc_bf16(dp, dsb);
    }
    {
      bf16x8 qta[2][4];
      to.read(qt, qta);
#pragma unroll
      for (int sg = 0; sg < 4; ++sg)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qta[dt][sg], dsb[sg], dk[dt], 0, 0, 0);
    }
  }

  // gradients of a padded key are exactly 0 (selected, not multiplied: its K row may hold anything)
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dk[dt][r] = key_valid ? dk[dt][r] * p.scale : 0.f;
      dv[dt][r] = key_valid ? (kDrop ? dv[dt][r] * p.drop.rs : dv[dt][r]) : 0.f;
    }
  store_acc_rows(dk_dst, dk, hf);
  store_acc_rows(dv_dst, dv, hf);
}

// ---------------------------------------------------------------------------------------
// Fixed-order sums of the partial gradients of split rows (dQ) and split columns (dK, dV)
// ---------------------------------------------------------------------------------------
// One launch covers all three: blocks [0, nq) are the dQ blocks of split query rows, then
// come the dK and the dV blocks of the global key blocks.  Four workgroups per 64x64 block,
// thread t owns 4 columns of row part*16 + t/16.
__global__ __launch_bounds__(256) void bwd_reduce_kernel(BwdParams p, int nq_blocks, int nkv_blocks) {
  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const int part = blockIdx.x & 3;
  int blk = blockIdx.x >> 2;
  const float* src;
  float* dst;
  int nslices;
  if (blk < nq_blocks) {
    const RowSplit& s = p.split;
    const int nglob_rows = s.cg > 1 ? p.g : 0;
    const int nsparse_rows = s.cs > 1 ? p.nb - p.g : 0;
    const int rows_per_bh = nglob_rows + nsparse_rows;
    const int bh = blk / rows_per_bh, rr = blk % rows_per_bh;
    int j, slot0;
    if (rr < nglob_rows) {
      j = pat.global_block(rr);
      nslices = s.cg;
      slot0 = bh * s.slots_per_bh + rr * s.cg;
    } else {
      const int t = rr - nglob_rows;
      j = pat.sparse_block(t);
      nslices = s.cs;
      slot0 = bh * s.slots_per_bh + (s.cg > 1 ? p.g * s.cg : 0) + t * s.cs;
    }
    src = p.part_dq + static_cast<size_t>(slot0) * (kBlk * kDim);
    dst = p.dQ + (static_cast<size_t>(bh) * p.n + j * kBlk) * kDim;
  } else {
    blk -= nq_blocks;
    const bool is_dv = blk >= nkv_blocks;
    if (is_dv) blk -= nkv_blocks;
    const int bh = blk / p.g, gi = blk % p.g;
    nslices = p.cq;
    const size_t slot0 = static_cast<size_t>(bh * p.g + gi) * p.cq;
    src = (is_dv ? p.part_dv : p.part_dk) + slot0 * (kBlk * kDim);
    dst = (is_dv ? p.dV : p.dK) + (static_cast<size_t>(bh) * p.n + pat.global_block(gi) * kBlk) * kDim;
  }
  const int off = (part * 16 + (threadIdx.x >> 4)) * kDim + (threadIdx.x & 15) * 4;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int U = 8;
  for (int c0 = 0; c0 < nslices; c0 += U) {
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cidx = c0 + u < nslices ? c0 + u : nslices - 1;
      v[u] = *reinterpret_cast<const f32x4*>(src + static_cast<size_t>(cidx) * (kBlk * kDim) + off);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (c0 + u < nslices) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += v[u][e];
      }
  }
  *reinterpret_cast<f32x4*>(dst + off) = acc;
}

namespace {
bool launch_failed(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return false;
  fprintf(stderr, "bigbird: launch of %s failed: %s\n", what, hipGetErrorString(e));
  return true;
}
}  // namespace

int launch_bwd_bf16(const BwdParams& p, hipStream_t stream) {
  const RowSplit& s = p.split;
  const unsigned qgrid = static_cast<unsigned>(kXcd) * s.bh_rounds * s.items_per_bh;
  const bool drop = p.drop.thr != 0;
  if (drop)
    hipLaunchKernelGGL(bwd_dq_kernel<true>, dim3(qgrid), dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL(bwd_dq_kernel<false>, dim3(qgrid), dim3(kThreads), 0, stream, p);
  if (launch_failed("bwd_dq_kernel")) return BB_ERR_LAUNCH;
  const unsigned kvgrid = static_cast<unsigned>(kXcd) * s.bh_rounds * p.kv_items_per_bh;
  if (drop)
    hipLaunchKernelGGL(bwd_dkv_kernel<true>, dim3(kvgrid), dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL(bwd_dkv_kernel<false>, dim3(kvgrid), dim3(kThreads), 0, stream, p);
  if (launch_failed("bwd_dkv_kernel")) return BB_ERR_LAUNCH;

  // one reduction launch for the split dQ rows and the split dK / dV columns
  const int rows_per_bh = (s.cg > 1 ? p.g : 0) + (s.cs > 1 ? p.nb - p.g : 0);
  const int nq_blocks = p.BH * rows_per_bh;
  const int nkv_blocks = (p.g > 0 && p.cq > 1) ? p.BH * p.g : 0;
  const int total = nq_blocks + 2 * nkv_blocks;
  if (total > 0) {
    hipLaunchKernelGGL(bwd_reduce_kernel, dim3(static_cast<unsigned>(total) * 4), dim3(256), 0, stream, p,
                       nq_blocks, nkv_blocks);
    if (launch_failed("bwd_reduce_kernel")) return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
