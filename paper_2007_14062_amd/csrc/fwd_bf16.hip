// bf16 forward kernel: the tuned path of the BERT-shaped workloads.
//
// Same mathematics as the fp32 kernel (eq. (AT) per head on the App. D pattern),
// organised around what limits it on this chip at d = 64: the vector ALU (one
// exponential per score) and the LDS read port (every MFMA wants a fresh 1 KB
// operand), not the matrix pipe.
//   * One wavefront owns one work item: a 64-query block against a slice of its key
//     blocks.  Waves never wait for each other inside the key-block loop.  A workgroup
//     is four such waves: either four consecutive non-global query blocks (independent
//     items), or one global query block whose key list is dealt out 16 blocks per wave
//     and merged in LDS at the end (no partial results in HBM, no second kernel, for
//     up to 64 key blocks; longer rows take several workgroups plus the merge kernel).
//   * The wave's queries form two 32-column MFMA tiles (A, B).  Every K and V^T
//     operand fetched from LDS feeds two MFMAs (one per tile), which halves the LDS
//     traffic per flop, and the tiles ping-pong: while the vector ALU exponentiates
//     tile A the matrix pipe computes tile B's scores; tile A's probabilities then wait
//     in registers and its share of P V runs under tile B's exponentials.  The issue
//     order (one MFMA, a handful of vector instructions, ...) is pinned with scheduling
//     group barriers: left alone the compiler issues the MFMAs back to back, and a wave
//     cannot issue anything else while it queues them.
//   * K and V tiles go global -> LDS directly (no registers in between), one 8 KB
//     buffer each: a tile is read out into operand registers in one burst and the
//     next block's load is issued at once, so it has a whole block of work to land.
//   * V^T operands come from the transposing LDS read; the LDS layout is swizzled so
//     that neither read pattern has bank conflicts.
//   * The softmax reference exponent moves only when a row maximum grows by more
//     than 2^8, so the accumulator rescale is rare; row sums are taken from the
//     bf16-rounded probabilities with the packed dot instruction.
#include "fwd_epilogue.h"
#include "tile_ops.h"

#include <cstdio>

namespace bb {

namespace {

constexpr float kLazyLog2 = 8.f;  // rescale when a row maximum grows by more than 2^8
constexpr int kFwdWaves = 4;
constexpr int kFwdThreads = 64 * kFwdWaves;  // four independent wavefronts, one work item each
constexpr int kTile = kBlk * kDim * 2;  // 8 KB

__device__ __forceinline__ void zero_acc(f32x16 (&a)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) a[t][r] = 0.f;
}

__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const uintptr_t v = reinterpret_cast<uintptr_t>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(v));
  const unsigned hi = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(v >> 32));
  return reinterpret_cast<const char*>((static_cast<uintptr_t>(hi) << 32) | lo);
}

// A whole 64x64 bf16 tile, global -> LDS, by one wave: eight instructions of 64 lanes x
// 16 bytes.  Instruction ii fills LDS rows 8*ii .. 8*ii+7 linearly (lane l lands on row
// l/8, chunk position l%8) and fetches, for that place, the chunk the swizzle stores
// there.  The swizzle depends on row bits 1..3, i.e. on l/8 and on the parity of ii:
// voff[0] / voff[1] are the per-lane byte offsets for even / odd ii.  The instruction's
// immediate offset moves the global and the LDS address alike, so four instructions
// share one base pair (M0, scalar address) and no vector arithmetic is needed.
__device__ __forceinline__ void tile_load_async_wave(const char* gtile_, unsigned lds, const unsigned (&voff)[2]) {
  const char* gtile = uniform_ptr(gtile_);  // wave-uniform by construction: keep it in scalar registers
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
    asm volatile(
        "s_mov_b32 m0, %3\n\t"
        "global_load_lds_dwordx4 %0, %2\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
        "global_load_lds_dwordx4 %0, %2 offset:2048\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:3072"
        :
        : "v"(voff[0]), "v"(voff[1]), "s"(gtile + hh * 4096), "s"(lds + hh * 4096)
        : "memory");  // M0 is written here; nothing else in this kernel reads M0
}

// Key-block list of a non-global row without a padding mask, from the row of the pattern table
// that lanes 0 .. r-1 already hold in `rnd` (one entry per lane).  Same candidate order and
// rules as build_key_list_range: global blocks, window blocks, random blocks; a candidate is
// dropped if an earlier component already holds it.  Entries [lo, lo+len) go to klist.
__device__ __forceinline__ int finish_key_list_sparse(const Pattern& pat, int r, int j, int rnd, int lo,
                                                       int len, int* klist) {
  const int lane = lane_id();
  const int nb = pat.nb;
  const int ncand = pat.g + pat.w + r;  // <= 64 (checked by the caller)
  bool valid = false;
  int k = -1;
  const int t = lane - pat.g - pat.w;
  const int mine = __shfl(rnd, t < 0 ? 0 : t);  // entry t of the row, for the lanes that stand for it
  if (lane < pat.g) {
    k = pat.global_block(lane);
    valid = true;
  } else if (lane < pat.g + pat.w) {
    k = j - pat.half() + (lane - pat.g);
    valid = k >= 0 && k < nb && !pat.is_global(k);
  } else if (lane < ncand) {
    k = mine;
    valid = k >= 0 && k < nb && !pat.is_global(k) && !pat.in_window(j, k);
  }
  for (int u = 0; u < r; ++u) {
    const int ku = __builtin_amdgcn_readlane(rnd, u);
    if (u < t && ku == k) valid = false;
  }
  const uint64_t m = __ballot(valid);
  const int rank = mask_rank(m);
  if (valid && rank >= lo && rank < lo + len) klist[rank - lo] = k;
  int cnt = static_cast<int>(__popcll(m)) - lo;
  return cnt < 0 ? 0 : (cnt > len ? len : cnt);
}

}  // namespace

__global__ __launch_bounds__(kFwdThreads) __attribute__((amdgpu_waves_per_eu(2)))
void fwd_kernel_bf16(FwdParams p) {
  __shared__ __attribute__((aligned(1024))) char lds_all[kFwdWaves][2 * kTile];  // per wave: K tile, V tile
  __shared__ int klist_all[kFwdWaves][kGlobalWaveLen];
  __shared__ float mrg_m[kFwdWaves][kBlk], mrg_l[kFwdWaves][kBlk];  // global rows: per-wave exponent, sum

  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const Bf16Geom& geo = p.geo;
  const int lane = lane_id(), wv = threadIdx.x >> 6;
  const int hf = lane >> 5, col = lane & 31;
  char* const lds_kv = lds_all[wv];
  char* const lds_k = lds_kv;
  char* const lds_v = lds_kv + kTile;
  int* const klist = klist_all[wv];

  // Workgroup id -> work.  id % 8 is the die (XCD) the hardware dispatches to; each die gets
  // whole (batch, head) slices so that a slice's K and V stay in its L2.  Within a die the
  // global-row workgroups of all its slices come first: they are the longest.
  WorkItem it;
  int list_lo, list_len;
  {
    const int xcd = blockIdx.x % kXcd;
    unsigned q = blockIdx.x / kXcd;
    const unsigned n_gpart = static_cast<unsigned>(geo.bh_rounds) * geo.g_wgs;
    if (q < n_gpart) {
      it.bh = (q / geo.g_wgs) * kXcd + xcd;
      const int gidx = q % geo.g_wgs;
      const int row = gidx / geo.ng, u = gidx % geo.ng;
      it.row_global = true;
      it.j = pat.global_block(row);
      it.chunk = u;
      it.nchunks = geo.ng;
      it.slot = it.bh * p.slots_per_bh + row * geo.ng + u;
      list_lo = (u * kFwdWaves + wv) * geo.gw_len;
      list_len = geo.gw_len;
      if (it.bh >= p.BH) return;  // whole workgroup
    } else {
      q -= n_gpart;
      it.bh = (q / geo.s_wgs) * kXcd + xcd;
      const int sitem = (q % geo.s_wgs) * kFwdWaves + wv;
      if (it.bh >= p.BH || sitem >= geo.n_sitems) return;  // no barrier follows for these workgroups
      it.row_global = false;
      it.j = pat.sparse_block(sitem / geo.cs);
      it.chunk = sitem % geo.cs;
      it.nchunks = geo.cs;
      it.slot = it.bh * p.slots_per_bh + p.cmb_g_rows * p.cmb_g_n + sitem;
      list_lo = it.chunk * kGlobalWaveLen;  // up to 16 key blocks per item (8 at the ITC base pattern)
      list_len = kGlobalWaveLen;
    }
  }
  const int bi = it.bh / p.H, h = it.bh % p.H;

  const size_t bh_row0 = static_cast<size_t>(it.bh) * p.n;
  const size_t qrow0 = bh_row0 + it.j * kBlk + col;  // tile A row of this lane; tile B is 32 rows on
  const char* kbase = static_cast<const char*>(p.K) + bh_row0 * (kDim * 2);
  const char* vbase = static_cast<const char*>(p.V) + bh_row0 * (kDim * 2);

  unsigned voff[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const int row = par * 8 + (lane >> 3);
    voff[par] = (lane >> 3) * 128 + (((lane & 7) ^ tile_swizzle(row)) << 4);
  }
  const unsigned lds_k_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_k));
  const unsigned lds_v_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_v));

  // The first key block is nearly always known before the list is: a global row's slice starts
  // at its own offset unless padding removed blocks before it, every other row starts with the
  // first global block.  Its tiles are asked for now, so that their flight overlaps the reads
  // of the pattern table instead of following them.
  // For a non-global row without a padding mask the pattern-table row is asked for before
  // anything else (one entry per lane, by inline asm so that it can be waited for by count:
  // loads return in order, and the tile and Q loads issued after it need not have landed when
  // the list is built).
  const bool fast_list = !it.row_global && !p.kmask && p.rand_idx && p.r > 0 && p.g + p.w + p.r <= 64;
  int rnd = -1;
  if (fast_list) {
    const int32_t* rrow = p.rand_idx + (static_cast<size_t>(h) * p.nb + it.j) * p.r + (lane < p.r ? lane : 0);
    asm volatile("global_load_dword %0, %1, off" : "=v"(rnd) : "v"(rrow) : "memory");
  }

  int spec = -1;
  if (it.row_global) {
    if (list_lo < p.nb) spec = list_lo;
  } else if (it.chunk == 0 && p.g > 0) {
    spec = pat.global_block(0);
  }
  if (spec >= 0) tile_load_async_wave(kbase + static_cast<size_t>(spec) * kTile, lds_k_a, voff);

  // The query block takes the same road as a key block: eight coalesced 1 KB loads into LDS
  // (the V buffer, idle until the first block's second half), then operand reads.  Register
  // loads of the operand layout would touch every row of the tile in each instruction and cost
  // the address unit four times as many cache-line requests.
  tile_load_async_wave(static_cast<const char*>(p.Q) + (bh_row0 + it.j * kBlk) * (kDim * 2), lds_v_a, voff);

  int cnt;
  if (fast_list) {
    // younger than the table load: the guessed K tile's 8 loads (if any) and Q's 8
    if (spec >= 0)
      asm volatile("s_waitcnt vmcnt(16)" : "+v"(rnd)::"memory");
    else
      asm volatile("s_waitcnt vmcnt(8)" : "+v"(rnd)::"memory");
    if (lane >= p.r) rnd = -1;
    cnt = finish_key_list_sparse(pat, p.r, it.j, rnd, list_lo, list_len, klist);
  } else {
    cnt = build_key_list_range(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, it.j, it.row_global, list_lo,
                               list_len, klist);
  }
  // same wave wrote and reads the list: LDS keeps a wave's accesses in order, the compiler must too
  asm volatile("" ::: "memory");
  const int kl = klist[lane & (kGlobalWaveLen - 1)];  // lane t holds list entry t % 16
  auto key_block = [&](int i) { return __builtin_amdgcn_readlane(kl, i); };
  auto tile_off = [&](int i) { return static_cast<size_t>(key_block(i)) * kTile; };

  // Q^T operands (B of S^T = K Q^T) of the two query tiles: lane holds query `col` (+32 for
  // tile B), d = 16*ks + 8*hf .. +8 -- the "straight" fragments of the Q tile.
  bf16x8 qb[2][4];
  const StraightOffsets so(lane);
  const bool guessed = cnt > 0 && key_block(0) == spec;
  if (!guessed && cnt > 0) {
    // wrong guess (or none): everything issued so far lands, then the right K tile is asked for
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    asm volatile("" ::: "memory");
    tile_load_async_wave(kbase + tile_off(0), lds_k_a, voff);
    so.read(lds_v, qb);
  } else {
    // Q was issued after the guessed K tile: when it has landed, so has K
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    asm volatile("" ::: "memory");
    so.read(lds_v, qb);
  }
  __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
  asm volatile("" ::: "memory");
  if (cnt > 0) tile_load_async_wave(vbase + tile_off(0), lds_v_a, voff);

  f32x16 o[2][2];  // [query tile][d tile]: O^T accumulators
  zero_acc(o[0]);
  zero_acc(o[1]);
  float m_ref[2] = {neg_inf(), neg_inf()};  // reference exponents, raw score units (halves agree)
  float l_run[2] = {0.f, 0.f};              // this lane's share of sum 2^((s - m_ref) c)
  const float c = p.c;
  const float tau = kLazyLog2 / c;
  const TransposedOffsets to(lane);
  const bf16x2 ones = {static_cast<__bf16>(1.f), static_cast<__bf16>(1.f)};

  for (int i = 0; i < cnt; ++i) {
    const bool more = i + 1 < cnt;
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, bi, p.n, key_block(i));
    size_t next_off = 0;
    if (more) next_off = tile_off(i + 1);

    // ---- K(i): wait for it (V(i)'s eight loads were issued later and may be in flight),
    // pull all its operand pieces into registers, then reuse the buffer for K(i+1)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
    asm volatile("" ::: "memory");
    bf16x8 ka[2][4];
    so.read(lds_k, ka);
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
    asm volatile("" ::: "memory");
    if (more) tile_load_async_wave(kbase + next_off, lds_k_a, voff);

    f32x16 s[2][2];
    auto scores = [&](int q, int ks) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (ks == 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s[q][t][r] = 0.f;
        }
        s[q][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t][ks], qb[q][ks], s[q][t], 0, 0, 0);
      }
    };
    auto mask_scores = [&](int q) {
      const uint64_t mine = vbits >> (hf * 4);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!((mine >> (t * 32 + acc_row(r, 0))) & 1)) s[q][t][r] = neg_inf();
    };
    // online softmax of tile q, base 2, lazily moved reference: returns the exponent offset
    auto tile_reference = [&](int q) {
      float mloc = neg_inf();
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[q][t][r]);
      mloc = half_max(mloc);
      if (__any(mloc > m_ref[q] + tau)) {
        const float m_new = fmaxf(m_ref[q], mloc);
        const float m_use = (m_new == neg_inf()) ? 0.f : m_new;
        const float alpha = fast_exp2((m_ref[q] - m_use) * c);
        l_run[q] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[q][dt][r] *= alpha;
        m_ref[q] = m_new;
      }
      return (m_ref[q] == neg_inf()) ? 0.f : m_ref[q] * c;
    };
    // probabilities of 16 keys (group sg) of tile q as a B operand; row sums on the side
    auto probs = [&](int q, int sg, float mc) {
      bf16x8 pb;
#pragma unroll
      for (int kk = 0; kk < 8; kk += 2) {
        const int t = sg >> 1, r = (sg & 1) * 8 + kk;
        const float p0 = fast_exp2(__builtin_fmaf(s[q][t][r], c, -mc));
        const float p1 = fast_exp2(__builtin_fmaf(s[q][t][r + 1], c, -mc));
        const bf16x2 pk = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
        pb[kk] = pk[0];
        pb[kk + 1] = pk[1];
        l_run[q] = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l_run[q], false);
      }
      return pb;
    };

    // ---- phase 1: scores of tile A
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) scores(0, ks);
    if (vbits != ~0ull) mask_scores(0);

    // ---- phase 2: tile A's exponentials on the vector ALU while the matrix pipe computes tile
    // B's scores; the probabilities wait in registers for V
    const float mc_a = tile_reference(0);
    bf16x8 pa[4];
#pragma unroll
    for (int sg = 0; sg < 4; ++sg) {
      scores(1, sg);
      pa[sg] = probs(0, sg, mc_a);
      asm volatile("" : "+v"(pa[sg]));  // computed here, not where it is used
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {  // issue order: one MFMA, a dozen vector instructions, ...
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 12, 0);
    }
    if (vbits != ~0ull) mask_scores(1);

    // ---- V(i): wait (K(i+1)'s loads, if any, are younger), fetch all V^T operand pieces
    if (more)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    asm volatile("" ::: "memory");
    bf16x8 va[2][4];
    to.read(lds_v, va);
    const float mc_b = tile_reference(1);
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
    asm volatile("" ::: "memory");
    if (more) tile_load_async_wave(vbase + next_off, lds_v_a, voff);

    // ---- phase 3: tile B's exponentials while the matrix pipe does tile A's share of
    // O^T += V^T P^T, then tile B's
#pragma unroll
    for (int sg = 0; sg < 4; ++sg) {
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        o[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt][sg], pa[sg], o[0][dt], 0, 0, 0);
      const bf16x8 pb = probs(1, sg, mc_b);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        o[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt][sg], pb, o[1][dt], 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 6, 0);
    }
  }

  // ---- finalise.  The accumulators hold O^T (a lane owns one query and scattered groups
  // of four d); they are turned through LDS (free now) so that global memory sees whole
  // rows: 16 bytes per lane, consecutive lanes on consecutive addresses.
  float l_tot[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) l_tot[q] = half_sum(l_run[q]);
  const size_t row_blk = bh_row0 + it.j * kBlk;  // first row of the query block
  if (!it.row_global && it.nchunks == 1) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const float inv = l_tot[q] > 0.f ? 1.f / l_tot[q] : 0.f;
      if (hf == 0)
        p.LSE[qrow0 + q * 32] = l_tot[q] > 0.f ? (m_ref[q] * c + fast_log2(l_tot[q])) * kLn2 : neg_inf();
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[q][dt][r4 * 4 + e] * inv);
          // d0 = 32 dt + 8 r4 + 4 hf: 16-byte chunk 4 dt + r4, upper or lower half of it
          *reinterpret_cast<bf16x4*>(lds_kv + tile_off_bf16(q * 32 + col, dt * 4 + r4) + hf * 8) = v;
        }
    }
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
    asm volatile("" ::: "memory");
    __bf16* orow = static_cast<__bf16*>(p.O) + row_blk * kDim;
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      const int row = ii * 8 + (lane >> 3), chunk = lane & 7;
      const u32x4 v = *reinterpret_cast<const u32x4*>(lds_kv + tile_off_bf16(row, chunk));
      *reinterpret_cast<u32x4*>(orow + row * kDim + chunk * 8) = v;
    }
    return;
  }

  // Un-normalised O of this wave as an fp32 [64 q][64 d] tile in its LDS region: d 0..31 in the
  // first 8 KB, d 32..63 in the second, each laid out like a bf16 tile (128-byte rows of 32 floats).
#pragma unroll
  for (int q = 0; q < 2; ++q)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = o[q][dt][r4 * 4 + e];
        *reinterpret_cast<f32x4*>(lds_kv + dt * kTile + tile_off_bf16(q * 32 + col, r4 * 2 + hf)) = v;
      }

  if (!it.row_global) {
    // slice of a non-global row with several slices: partial triple for the merge kernel
    float* pml = p.part_ml + static_cast<size_t>(it.slot) * (2 * kBlk);
#pragma unroll
    for (int q = 0; q < 2; ++q)
      if (hf == 0) {
        pml[q * 32 + col] = (m_ref[q] == neg_inf()) ? neg_inf() : m_ref[q] * c;
        pml[kBlk + q * 32 + col] = l_tot[q];
      }
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
    asm volatile("" ::: "memory");
    float* po = p.part_o + static_cast<size_t>(it.slot) * (kBlk * kDim);
#pragma unroll
    for (int ii = 0; ii < 16; ++ii) {
      const int row = ii * 4 + (lane >> 4), cc = lane & 15;
      const f32x4 v = *reinterpret_cast<const f32x4*>(lds_kv + (cc >> 3) * kTile + tile_off_bf16(row, cc & 7));
      *reinterpret_cast<f32x4*>(po + row * kDim + cc * 4) = v;
    }
    return;
  }

  // ---- global row: merge the four waves' (m, l, O~) in LDS.  Wave w then owns query rows
  // 16w .. 16w+15; a lane owns 16 d columns of one row.
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (hf == 0) {
      mrg_m[wv][q * 32 + col] = (m_ref[q] == neg_inf() || !(l_tot[q] > 0.f)) ? neg_inf() : m_ref[q] * c;
      mrg_l[wv][q * 32 + col] = l_tot[q];
    }
  __syncthreads();  // all four waves of a global workgroup arrive here
  {
    const int q = wv * 16 + (lane >> 2), part = lane & 3;
    float M = neg_inf();
#pragma unroll
    for (int v = 0; v < kFwdWaves; ++v) M = fmaxf(M, mrg_m[v][q]);
    f32x4 acc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    float L = 0.f;
    if (M != neg_inf()) {
#pragma unroll
      for (int v = 0; v < kFwdWaves; ++v) {
        const float mv = mrg_m[v][q];
        const float wgt = (mv == neg_inf()) ? 0.f : fast_exp2(mv - M);
        L += mrg_l[v][q] * wgt;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int cc = part * 4 + e;
          const f32x4 x =
              *reinterpret_cast<const f32x4*>(lds_all[v] + (cc >> 3) * kTile + tile_off_bf16(q, cc & 7));
#pragma unroll
          for (int z = 0; z < 4; ++z) acc[e][z] += x[z] * wgt;
        }
      }
    }
    const size_t row = row_blk + q;
    if (it.nchunks == 1) {
      const float inv = L > 0.f ? 1.f / L : 0.f;
      if (part == 0) p.LSE[row] = L > 0.f ? (M + fast_log2(L)) * kLn2 : neg_inf();
      bf16x8 v0, v1;
#pragma unroll
      for (int z = 0; z < 4; ++z) {
        v0[z] = static_cast<__bf16>(acc[0][z] * inv);
        v0[4 + z] = static_cast<__bf16>(acc[1][z] * inv);
        v1[z] = static_cast<__bf16>(acc[2][z] * inv);
        v1[4 + z] = static_cast<__bf16>(acc[3][z] * inv);
      }
      bf16x8* dst = reinterpret_cast<bf16x8*>(static_cast<__bf16*>(p.O) + row * kDim + part * 16);
      dst[0] = v0;
      dst[1] = v1;
    } else {
      // one of several workgroups of a long global row: merged partial triple for the merge kernel
      float* pml = p.part_ml + static_cast<size_t>(it.slot) * (2 * kBlk);
      if (part == 0) {
        pml[q] = L > 0.f ? M : neg_inf();
        pml[kBlk + q] = L;
      }
      f32x4* dst =
          reinterpret_cast<f32x4*>(p.part_o + static_cast<size_t>(it.slot) * (kBlk * kDim) + q * kDim + part * 16);
#pragma unroll
      for (int e = 0; e < 4; ++e) dst[e] = acc[e];
    }
  }
}

int launch_fwd_bf16_main(const FwdParams& p, hipStream_t stream) {
  const unsigned grid = static_cast<unsigned>(kXcd) * p.geo.bh_rounds * (p.geo.g_wgs + p.geo.s_wgs);
  if (grid == 0) return BB_OK;
  hipLaunchKernelGGL(fwd_kernel_bf16, dim3(grid), dim3(kFwdThreads), 0, stream, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    fprintf(stderr, "bigbird: launch of fwd_kernel_bf16 failed: %s\n", hipGetErrorString(e));
    return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
