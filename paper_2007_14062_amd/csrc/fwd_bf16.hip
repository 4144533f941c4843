// bf16 forward kernel: the tuned path of the BERT-shaped workloads.
//
// Same mathematics as the fp32 kernel (eq. (AT) per head on the App. D pattern),
// organised around what limits it on this chip at d = 64: the vector ALU (one
// exponential per score), the LDS port and the matrix pipe are all within a factor of
// two of each other, so every vector instruction per score counts.
//   * One wavefront owns one work item: a 64-query block against a slice of its key
//     blocks.  Waves never wait for each other inside the key-block loop.  A workgroup
//     is four such waves: either four consecutive non-global query blocks (independent
//     items), or one global query block whose key list is dealt out 16 blocks per wave
//     and merged in LDS at the end (no partial results in HBM, no second kernel, for
//     up to 64 key blocks; longer rows take several workgroups plus the merge kernel).
//   * Softmax without a running maximum.  The query fragments are multiplied by
//     scale*log2(e) once per item (and rounded to bf16 again), so a score leaves the MFMA
//     as the base-2 exponent and a probability is one v_exp_f32: no multiply-add, no row
//     maximum, no accumulator rescale.  Softmax is shift invariant and fp32/bf16 carry
//     eight exponent bits, so a fixed reference of 0 is exact as long as the row sum stays
//     inside [2^-40, 2^60]; a wave checks that at the end of its item and, if a row left
//     the range (logits beyond about +-28 in natural units), recomputes the item with the
//     classical running-maximum recurrence (slow_item).  Both paths give the same
//     un-normalised (reference, sum, O~) triple to the common epilogue.
//   * The block pair is cut into four units (32 keys x 32 queries each) that flow through
//     a three-stage software pipeline inside the wave: scores of unit u+1 on the matrix
//     pipe, exponentials of unit u on the vector ALU, P V of unit u-1 on the matrix pipe
//     again.  The pipeline runs across key-block boundaries; its first and last pairs
//     are separate instantiations, so every loop body is straight-line code whose issue
//     order (one MFMA, four vector instructions, ...) is pinned with scheduling group
//     barriers.  Every K and V^T operand fetched from LDS feeds two MFMAs (two query
//     tiles), which halves the LDS traffic per flop.
//   * K and V tiles go global -> LDS directly (no registers in between), one 8 KB
//     buffer each, handled as 32-key halves: as soon as a half has been read out into
//     operand registers the same half of the next key block is requested, so a load has
//     three quarters of a block pair to land.
//   * V^T operands come from the transposing LDS read; the LDS layout is swizzled so
//     that neither read pattern has bank conflicts.
#include "fwd_epilogue.h"
#include "tile_ops.h"

#include <cstdio>

namespace bb {

namespace {

constexpr int kFwdWaves = 4;
constexpr int kFwdThreads = 64 * kFwdWaves;  // four independent wavefronts, one work item each
constexpr int kTile = kBlk * kDim * 2;       // 8 KB
constexpr int kHalfTile = kTile / 2;         // 32 rows

// Row sums of the reference-free path must stay inside [kSumLo, kSumHi] (see the file header).
constexpr float kSumLo = 0x1p-40f;
constexpr float kSumHi = 0x1p60f;

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

// Half of a 64x64 bf16 tile (rows 32*hh .. +32), global -> LDS, by one wave: four
// instructions of 64 lanes x 16 bytes.  Instruction ii fills LDS rows 8*ii .. 8*ii+7 of
// the half linearly (lane l lands on row l/8, chunk position l%8) and fetches, for that
// place, the chunk the swizzle stores there.  The swizzle depends on row bits 1..3, i.e. on
// l/8 and on the parity of ii: voff[0] / voff[1] are the per-lane byte offsets for even /
// odd ii.  The instruction's immediate offset moves the global and the LDS address alike,
// so the four instructions share one base pair (M0, scalar address).
__device__ __forceinline__ void half_load_async(const char* gtile, unsigned lds, int hh,
                                                const unsigned (&voff)[2]) {
  asm volatile(
      "s_mov_b32 m0, %3\n\t"
      "s_nop 0\n\t"  // a scalar write of M0 needs one wait state before an LDS-DMA load reads it
      "global_load_lds_dwordx4 %0, %2\n\t"
      "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
      "global_load_lds_dwordx4 %0, %2 offset:2048\n\t"
      "global_load_lds_dwordx4 %1, %2 offset:3072"
      :
      : "v"(voff[0]), "v"(voff[1]), "s"(gtile + hh * kHalfTile), "s"(lds + hh * kHalfTile)
      : "memory");  // M0 is written here; it is a reserved register that the compiler only sets right before
                    // instructions of its own that read it, and this kernel has none
}

__device__ __forceinline__ void tile_load_async_wave(const char* gtile_, unsigned lds, const unsigned (&voff)[2]) {
  const char* gtile = uniform_ptr(gtile_);  // wave-uniform by construction: keep it in scalar registers
  half_load_async(gtile, lds, 0, voff);
  half_load_async(gtile, lds, 1, voff);
}

// One entry of a pattern-table row per lane, requested ahead of a whole tile (global -> LDS as in
// half_load_async) and waited for while the tile's eight loads stay in flight: loads return in
// order, so "all but the eight youngest" is exactly the table entry.  Request, tile loads and wait
// sit in one asm statement: the compiler sees the register only once the value is in it.
__device__ __forceinline__ int table_entry_then_tile(const int32_t* entry, const char* gtile_, unsigned lds,
                                                     const unsigned (&voff)[2]) {
  const char* gtile = uniform_ptr(gtile_);
  int e;
  asm volatile(
      "global_load_dword %0, %1, off\n\t"
      "s_mov_b32 m0, %5\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %4\n\t"
      "global_load_lds_dwordx4 %3, %4 offset:1024\n\t"
      "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
      "global_load_lds_dwordx4 %3, %4 offset:3072\n\t"
      "s_mov_b32 m0, %7\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %6\n\t"
      "global_load_lds_dwordx4 %3, %6 offset:1024\n\t"
      "global_load_lds_dwordx4 %2, %6 offset:2048\n\t"
      "global_load_lds_dwordx4 %3, %6 offset:3072\n\t"
      "s_waitcnt vmcnt(8)"
      : "=&v"(e)
      : "v"(entry), "v"(voff[0]), "v"(voff[1]), "s"(gtile), "s"(lds), "s"(gtile + kHalfTile), "s"(lds + kHalfTile)
      : "memory");
  return e;
}

// Waits and compiler fences.  The tile loads are invisible to the compiler's wait-count
// bookkeeping (inline asm), so every wait for them is written out; loads return in order,
// which makes "all but the N youngest" exact.
template <int N>
__device__ __forceinline__ void wait_tile_loads() {
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(N));
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void wait_lds_reads() {
  __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
  asm volatile("" ::: "memory");
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

// ---------------------------------------------------------------------------------------------
// The pipelined pair step.
//
// A block pair (64 queries x 64 keys) is four units u = (t, q): keys 32t .. 32t+31 against the
// query tile q (A: queries 0..31, B: 32..63), taken in the order (0,A) (0,B) (1,A) (1,B).
// Stage S(u): 4 MFMAs, S^T = K_t Q_q^T (keys along MFMA rows, a lane owns one query column).
// Stage E(u): 16 exponentials, 8 conversions to bf16 pairs, 8 packed dots for the row sum.
// Stage P(u): 4 MFMAs, O_q^T += V_t^T P^T, the converted scores being the B operand as they are.
// Slot k of the stream issues S(k+1), E(k), P(k-1).  Unit (0,A) of the next pair is therefore
// started in the last slot of this one, and P of unit (1,B) is finished in the first slot of
// the next pair (`sA`, `p3` carry them across).
//
// Operand registers: ka[t] (K half t, "straight" fragments), va[t] (V half t, transposed
// fragments).  Each is refilled from LDS in the slot after its last use, from the half tile that
// was requested three slots earlier; the request for the half after that follows as soon as the
// read has returned.  Tile loads outstanding at the start of a pair, oldest first:
// K(i+1).t0 and V(i).t1 (8 instructions).
//   FIRST: no pair precedes (nothing to finish for it).
//   TAIL : 0 = at least two more pairs follow, 1 = exactly one, 2 = none.
// Blocks with padded keys inside never come here: such items take the slow path.
struct PairCtx {
  const char* kbase;   // K, V of this (batch, head)
  const char* vbase;
  const char* lds_k;   // this wave's K and V tile buffers
  const char* lds_v;
  unsigned lds_k_a, lds_v_a;  // the same as LDS byte addresses (scalar)
  unsigned voff[2];
  int hf;
};

__device__ __forceinline__ void read_k_half(const StraightOffsets& so, const char* tile, int t, bf16x8 (&f)[4]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) f[ks] = *reinterpret_cast<const bf16x8*>(tile + so.off[ks] + t * kHalfTile);
}

__device__ __forceinline__ void read_v_half(const TransposedOffsets& to, const char* tile, int t,
                                            bf16x8 (&f)[2][2]) {
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int sgl = 0; sgl < 2; ++sgl) f[dt][sgl] = to.read_one(tile, dt, 2 * t + sgl);
}

__device__ __forceinline__ void unit_scores(const bf16x8 (&k)[4], const bf16x8 (&q)[4], f32x16& s) {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k[0], q[0], z, 0, 0, 0);
#pragma unroll
  for (int ks = 1; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k[ks], q[ks], s, 0, 0, 0);
}

__device__ __forceinline__ void unit_pv(const bf16x8 (&v)[2][2], const bf16x8 (&pb)[2], f32x16 (&o)[2]) {
#pragma unroll
  for (int sgl = 0; sgl < 2; ++sgl)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v[dt][sgl], pb[sgl], o[dt], 0, 0, 0);
}

// Probabilities of one unit as two B operands (16 keys each).  This lane's share of the row sum
// is taken from the unrounded values with plain additions, two chains: the packed bf16 dot
// instruction would halve the count, but it runs on the matrix pipe's data path and stalls
// against the MFMAs in flight (measured: 16 cycles per dot beside MFMAs, 4 per addition).
__device__ __forceinline__ void unit_probs(const f32x16& s, bf16x8 (&pb)[2], float (&l_run)[2]) {
#pragma unroll
  for (int sgl = 0; sgl < 2; ++sgl)
#pragma unroll
    for (int kk = 0; kk < 8; kk += 2) {
      const int r = sgl * 8 + kk;
      const float p0 = fast_exp2(s[r]);
      const float p1 = fast_exp2(s[r + 1]);
      const bf16x2 pk = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
      pb[sgl][kk] = pk[0];
      pb[sgl][kk + 1] = pk[1];
      l_run[0] += p0;
      l_run[1] += p1;
    }
}

// issue order of one slot: eight times (one MFMA, [LDS reads,] four vector instructions); nothing
// moves across the end of a slot
template <int DS_READS>
__device__ __forceinline__ void pin_slot() {
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (u * 2 < DS_READS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);  // two exponentials
    __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // their conversion and row-sum steps
  }
  __builtin_amdgcn_sched_barrier(0);
}

#ifdef BB_EXP_NOLOAD
#define half_load_async(...) ((void)0)
#define wait_tile_loads wait_nothing
template <int N> __device__ __forceinline__ void wait_nothing() {}
#endif
#ifdef BB_EXP_NOWAIT
#define wait_tile_loads wait_nothing
template <int N> __device__ __forceinline__ void wait_nothing() {}
#endif
// One block pair.  more1 / more2: one / two further pairs follow in this item (wave uniform).
// The arithmetic is the same for every pair of an item, so that one straight-line body serves
// them all: the first pair finishes a predecessor that does not exist (p3 = 0 on entry, V
// fragments zeroed), the last one starts a successor that does not exist (scores of stale K
// fragments, never used) -- eight idle MFMAs per item instead of six differently scheduled
// copies of the body.  Only the tile requests and the counts waited for depend on what follows;
// they sit at the slot boundaries behind scalar branches.
__device__ __forceinline__ void pair_step(const PairCtx& cx, const StraightOffsets& so, const TransposedOffsets& to,
                                          const bf16x8 (&qb)[2][4], bf16x8 (&ka)[2][4], bf16x8 (&va)[2][2][2],
                                          f32x16& sA, bf16x8 (&p3)[2], f32x16 (&o)[2][2], float (&l_run)[2][2],
                                          bool more1, bool more2, size_t off1, size_t off2) {
  f32x16 sB, sC, sD;
  bf16x8 p0[2], p1[2], p2[2];

  // ---- slot 0: the reads issued in the previous slot (K.t1, V.t0 of this pair) have returned
  wait_lds_reads();
  if (more1) {
    half_load_async(cx.kbase + off1, cx.lds_k_a, 1, cx.voff);
    half_load_async(cx.vbase + off1, cx.lds_v_a, 0, cx.voff);
  }
  unit_scores(ka[0], qb[1], sB);
  unit_pv(va[1], p3, o[1]);
  unit_probs(sA, p0, l_run[0]);
  pin_slot<0>();

  // ---- slot 1: K(i+1).t0 and V(i).t1 have landed
  if (more1) wait_tile_loads<8>(); else wait_tile_loads<0>();
  read_k_half(so, cx.lds_k, 0, ka[0]);
  read_v_half(to, cx.lds_v, 1, va[1]);
  unit_scores(ka[1], qb[0], sC);
  unit_pv(va[0], p0, o[0]);
  unit_probs(sB, p1, l_run[1]);
  pin_slot<12>();

  // ---- slot 2
  wait_lds_reads();
  if (more2) half_load_async(cx.kbase + off2, cx.lds_k_a, 0, cx.voff);
  if (more1) half_load_async(cx.vbase + off1, cx.lds_v_a, 1, cx.voff);
  unit_scores(ka[1], qb[1], sD);
  unit_pv(va[0], p1, o[1]);
  unit_probs(sC, p2, l_run[0]);
  pin_slot<0>();

  // ---- slot 3: K(i+1).t1 and V(i+1).t0 have landed
  if (more2) wait_tile_loads<8>(); else if (more1) wait_tile_loads<4>();
  read_k_half(so, cx.lds_k, 1, ka[1]);
  read_v_half(to, cx.lds_v, 0, va[0]);
  unit_scores(ka[0], qb[0], sA);
  unit_pv(va[1], p2, o[0]);
  unit_probs(sD, p3, l_run[1]);
  pin_slot<12>();
}

#ifdef BB_EXP_NOLOAD
#undef half_load_async
#undef wait_tile_loads
#endif
#ifdef BB_EXP_NOWAIT
#undef wait_tile_loads
#endif
#ifdef BB_EXP_NOLDS
#undef read_k_half
#undef read_v_half
#endif
// The item's block pairs through the pipeline.  On entry: K(0) is in the K buffer, V(0).t0 in
// flight or landed (4 loads, the oldest outstanding), nothing else outstanding.
__device__ __forceinline__ void fast_item(const PairCtx& cx, const StraightOffsets& so, const TransposedOffsets& to,
                                          const bf16x8 (&qb)[2][4], int cnt, int kl, f32x16 (&o)[2][2],
                                          float (&l_run)[2], long long* stamp = nullptr) {
  auto tile_off = [&](int i) { return static_cast<size_t>(__builtin_amdgcn_readlane(kl, i)) * kTile; };
  bf16x8 ka[2][4], va[2][2][2], p3[2];
  f32x16 sA;
  float lr[2][2] = {{0.f, 0.f}, {0.f, 0.f}};  // [query tile][chain]
#pragma unroll
  for (int a = 0; a < 2; ++a) {  // what the first pair "finishes": nothing
#pragma unroll
    for (int e = 0; e < 8; ++e) p3[a][e] = static_cast<__bf16>(0.f);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) va[1][a][b][e] = static_cast<__bf16>(0.f);
  }
  // start of the stream: K(0) -> registers, then the loads a pair expects to find outstanding
  read_k_half(so, cx.lds_k, 0, ka[0]);
  read_k_half(so, cx.lds_k, 1, ka[1]);
  wait_lds_reads();
  if (cnt > 1) half_load_async(cx.kbase + tile_off(1), cx.lds_k_a, 0, cx.voff);
  half_load_async(cx.vbase + tile_off(0), cx.lds_v_a, 1, cx.voff);
  if (cnt > 1) wait_tile_loads<8>(); else wait_tile_loads<4>();
  read_v_half(to, cx.lds_v, 0, va[0]);
  unit_scores(ka[0], qb[0], sA);
#ifdef BB_STAMPS
  stamp[5] = __builtin_readcyclecounter();
#endif

  for (int i = 0; i < cnt; ++i) {
    const bool more1 = i + 1 < cnt, more2 = i + 2 < cnt;
    pair_step(cx, so, to, qb, ka, va, sA, p3, o, lr, more1, more2, more1 ? tile_off(i + 1) : 0,
              more2 ? tile_off(i + 2) : 0);
  }
  // the last unit's share of O
  unit_pv(va[1], p3, o[1]);
#pragma unroll
  for (int q = 0; q < 2; ++q) l_run[q] = lr[q][0] + lr[q][1];
}

// The classical recurrence (running maximum, rescale on every block), one block pair at a time
// with synchronous tile loads: the fallback for items whose row sums left the safe range of the
// reference-free path.  Scores are base-2 exponents already (the query fragments carry the
// scale).  Leaves m_ref (exponent units), this lane's share of the row sums and O~.
__device__ __forceinline__ void slow_item(const PairCtx& cx, const StraightOffsets& so, const TransposedOffsets& to,
                                          const bf16x8 (&qb)[2][4], int cnt, int kl, int vlo, int vhi, bool masked,
                                          f32x16 (&o)[2][2], float (&l_run)[2], float (&m_ref)[2]) {
  const bf16x2 ones = {static_cast<__bf16>(1.f), static_cast<__bf16>(1.f)};
  zero_acc(o[0]);
  zero_acc(o[1]);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    m_ref[q] = neg_inf();
    l_run[q] = 0.f;
  }
  for (int i = 0; i < cnt; ++i) {
    const size_t off = static_cast<size_t>(__builtin_amdgcn_readlane(kl, i)) * kTile;
    uint64_t vbits = ~0ull;
    if (masked)
      vbits = (static_cast<uint64_t>(static_cast<unsigned>(__builtin_amdgcn_readlane(vhi, i))) << 32) |
              static_cast<unsigned>(__builtin_amdgcn_readlane(vlo, i));
    half_load_async(cx.kbase + off, cx.lds_k_a, 0, cx.voff);
    half_load_async(cx.kbase + off, cx.lds_k_a, 1, cx.voff);
    half_load_async(cx.vbase + off, cx.lds_v_a, 0, cx.voff);
    half_load_async(cx.vbase + off, cx.lds_v_a, 1, cx.voff);
    wait_tile_loads<0>();
    bf16x8 ka[2][4], va[2][2][2];
    read_k_half(so, cx.lds_k, 0, ka[0]);
    read_k_half(so, cx.lds_k, 1, ka[1]);
    read_v_half(to, cx.lds_v, 0, va[0]);
    read_v_half(to, cx.lds_v, 1, va[1]);
    wait_lds_reads();  // the buffers are overwritten by the next iteration's loads
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      f32x16 s[2];
      unit_scores(ka[0], qb[q], s[0]);
      unit_scores(ka[1], qb[q], s[1]);
      float mloc = neg_inf();
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const unsigned mine = static_cast<unsigned>(vbits >> (32 * t + cx.hf * 4));
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (!((mine >> acc_row(r, 0)) & 1)) s[t][r] = neg_inf();
          mloc = fmaxf(mloc, s[t][r]);
        }
      }
      mloc = half_max(mloc);
      const float m_new = fmaxf(m_ref[q], mloc);
      const float m_use = (m_new == neg_inf()) ? 0.f : m_new;
      const float alpha = fast_exp2(m_ref[q] - m_use);  // 0 while m_ref is still -inf
      l_run[q] *= alpha;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[q][dt][r] *= alpha;
      m_ref[q] = m_new;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 pb[2];
#pragma unroll
        for (int sgl = 0; sgl < 2; ++sgl)
#pragma unroll
          for (int kk = 0; kk < 8; kk += 2) {
            const int r = sgl * 8 + kk;
            const bf16x2 pk = {static_cast<__bf16>(fast_exp2(s[t][r] - m_use)),
                               static_cast<__bf16>(fast_exp2(s[t][r + 1] - m_use))};
            pb[sgl][kk] = pk[0];
            pb[sgl][kk + 1] = pk[1];
            l_run[q] = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l_run[q], false);
          }
        unit_pv(va[t], pb, o[q]);
      }
    }
  }
}

// Query fragments times scale*log2(e), rounded to bf16 again.
__device__ __forceinline__ void scale_fragments(bf16x8 (&f)[2][4], float c) {
#pragma unroll
  for (int q = 0; q < 2; ++q)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) f[q][ks][e] = static_cast<__bf16>(static_cast<float>(f[q][ks][e]) * c);
}

}  // namespace

__global__ __launch_bounds__(kFwdThreads) __attribute__((amdgpu_waves_per_eu(2)))
void fwd_kernel_bf16(FwdParams p) {
  __shared__ __attribute__((aligned(1024))) char lds_all[kFwdWaves][2 * kTile];  // per wave: K tile, V tile
  __shared__ int klist_all[kFwdWaves][kGlobalWaveLen];
  __shared__ float mrg_m[kFwdWaves][kBlk], mrg_l[kFwdWaves][kBlk];  // global rows: per-wave exponent, sum

#ifdef BB_STAMPS
  // development build: per-wave time stamps (shader clock) into the partial-result workspace
  long long stamp[6] = {0, 0, 0, 0, 0, 0};
  const long long rt0 = __builtin_amdgcn_s_memrealtime();
  stamp[0] = __builtin_readcyclecounter();
#define BB_STAMP(i) stamp[i] = __builtin_readcyclecounter()
#else
#define BB_STAMP(i)
#endif
  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const Bf16Geom& geo = p.geo;
  const int lane = lane_id();
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, and the compiler should know
  const int hf = lane >> 5, col = lane & 31;
  char* const lds_kv = lds_all[wv];
  char* const lds_k = lds_kv;
  char* const lds_v = lds_kv + kTile;
  int* const klist = klist_all[wv];

  // Workgroup id -> work.  id % 8 is the die (XCD) the hardware dispatches to; each die gets
  // whole (batch, head) slices so that a slice's K and V stay in its L2.  Within a die the
  // global-row workgroups of all its slices come first: they are the longest (running them
  // beside their own slice's other rows instead was measured 8 % slower).
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

  PairCtx cx;
  cx.kbase = uniform_ptr(static_cast<const char*>(p.K) + bh_row0 * (kDim * 2));
  cx.vbase = uniform_ptr(static_cast<const char*>(p.V) + bh_row0 * (kDim * 2));
  cx.lds_k = lds_k;
  cx.lds_v = lds_v;
  cx.hf = hf;
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const int row = par * 8 + (lane >> 3);
    cx.voff[par] = (lane >> 3) * 128 + (((lane & 7) ^ tile_swizzle(row)) << 4);
  }
  cx.lds_k_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_k));
  cx.lds_v_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_v));

  // The first key block is nearly always known before the list is: a global row's slice starts
  // at its own offset unless padding removed blocks before it, every other row starts with the
  // first global block.  Its tiles are asked for now, so that their flight overlaps the reads
  // of the pattern table instead of following them.
  // For a non-global row without a padding mask the row of the pattern table (one entry per
  // lane) is asked for before anything else and waited for while the first tile is in flight,
  // so the list is built under the flight of the tiles instead of after it.
  const bool fast_list = !it.row_global && !p.kmask && p.rand_idx && p.r > 0 && p.g + p.w + p.r <= 64;
  const int32_t* rentry = p.rand_idx + (static_cast<size_t>(h) * p.nb + it.j) * p.r + (lane < p.r ? lane : 0);
  const char* qtile = static_cast<const char*>(p.Q) + (bh_row0 + it.j * kBlk) * (kDim * 2);

  int spec = -1;
  if (it.row_global) {
    if (list_lo < p.nb) spec = list_lo;
  } else if (it.chunk == 0 && p.g > 0) {
    spec = pat.global_block(0);
  }
  // The query block takes the same road as a key block: eight coalesced 1 KB loads into LDS
  // (the V buffer, idle until the first block's second half), then operand reads.  Register
  // loads of the operand layout would touch every row of the tile in each instruction and cost
  // the address unit four times as many cache-line requests.
  int rnd = -1;
  if (spec >= 0) {
    const char* ktile = cx.kbase + static_cast<size_t>(spec) * kTile;
    if (fast_list)
      rnd = table_entry_then_tile(rentry, ktile, cx.lds_k_a, cx.voff);
    else
      tile_load_async_wave(ktile, cx.lds_k_a, cx.voff);
    tile_load_async_wave(qtile, cx.lds_v_a, cx.voff);
  } else if (fast_list) {
    rnd = table_entry_then_tile(rentry, qtile, cx.lds_v_a, cx.voff);
  } else {
    tile_load_async_wave(qtile, cx.lds_v_a, cx.voff);
  }

  int cnt;
  if (fast_list) {
    if (lane >= p.r) rnd = -1;
    cnt = finish_key_list_sparse(pat, p.r, it.j, rnd, list_lo, list_len, klist);
  } else {
    cnt = build_key_list_range(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, it.j, it.row_global, list_lo,
                               list_len, klist);
  }
  // same wave wrote and reads the list: LDS keeps a wave's accesses in order, the compiler must too
  asm volatile("" ::: "memory");
  const int kl = klist[lane & (kGlobalWaveLen - 1)];  // lane t holds list entry t % 16

  // Validity bits of the listed key blocks: lane t holds those of list entry t (two registers).
  // Read once per item, before the loop: a compiler-tracked load inside the loop would drain
  // the tile loads in flight.
  int vlo = -1, vhi = -1;
  bool any_partial = false;
  if (p.kmask) {
    for (int i = 0; i < cnt; ++i) {
      const uint64_t vb = key_valid_bits(p.kmask, bi, p.n, __builtin_amdgcn_readlane(kl, i));
      if (lane == i) {
        vlo = static_cast<int>(static_cast<unsigned>(vb));
        vhi = static_cast<int>(static_cast<unsigned>(vb >> 32));
      }
      any_partial |= vb != ~0ull;
    }
  }

  // Q^T operands (B of S^T = K Q^T) of the two query tiles: lane holds query `col` (+32 for
  // tile B), d = 16*ks + 8*hf .. +8 -- the "straight" fragments of the Q tile.
  bf16x8 qb[2][4];
  const StraightOffsets so(lane);
  const TransposedOffsets to(lane);
  const bool guessed = cnt > 0 && __builtin_amdgcn_readlane(kl, 0) == spec;
  wait_tile_loads<0>();  // Q was issued after the guessed K tile: when it has landed, so has K
  if (!guessed && cnt > 0)  // wrong guess (or none): the right K tile is asked for now
    tile_load_async_wave(cx.kbase + static_cast<size_t>(__builtin_amdgcn_readlane(kl, 0)) * kTile, cx.lds_k_a, cx.voff);
  so.read(lds_v, qb);
  wait_lds_reads();
  if (cnt > 0)
    half_load_async(cx.vbase + static_cast<size_t>(__builtin_amdgcn_readlane(kl, 0)) * kTile, cx.lds_v_a, 0, cx.voff);
  scale_fragments(qb, p.c);

  BB_STAMP(1);
  f32x16 o[2][2];  // [query tile][d tile]: O^T accumulators
  zero_acc(o[0]);
  zero_acc(o[1]);
  float m_ref[2] = {0.f, 0.f};  // reference exponents (base-2 units); halves agree
  float l_run[2] = {0.f, 0.f};  // this lane's share of sum 2^(s - m_ref)
  float l_tot[2] = {0.f, 0.f};
  if (cnt > 0) {
    if (!guessed) wait_tile_loads<4>();  // the K tile asked for late; V(0).t0 may still fly
    bool bad = any_partial;  // per-key masking is only in the slow path
    if (!any_partial) {
      BB_STAMP(2);
#ifdef BB_STAMPS
      fast_item(cx, so, to, qb, cnt, kl, o, l_run, stamp);
#else
      fast_item(cx, so, to, qb, cnt, kl, o, l_run);
#endif
      BB_STAMP(3);
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        l_tot[q] = half_sum(l_run[q]);
        bad |= !(l_tot[q] >= kSumLo && l_tot[q] <= kSumHi);
      }
    }
    if (__any(bad)) {
      slow_item(cx, so, to, qb, cnt, kl, vlo, vhi, p.kmask != nullptr, o, l_run, m_ref);
#pragma unroll
      for (int q = 0; q < 2; ++q) l_tot[q] = half_sum(l_run[q]);
    }
  } else {
    m_ref[0] = m_ref[1] = neg_inf();
  }

  // ---- finalise.  The accumulators hold O^T (a lane owns one query and scattered groups
  // of four d); they are turned through LDS (free now) so that global memory sees whole
  // rows: 16 bytes per lane, consecutive lanes on consecutive addresses.
  const size_t row_blk = bh_row0 + it.j * kBlk;  // first row of the query block
  if (!it.row_global && it.nchunks == 1) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const float inv = l_tot[q] > 0.f ? 1.f / l_tot[q] : 0.f;
      if (hf == 0)
        p.LSE[qrow0 + q * 32] = l_tot[q] > 0.f ? (m_ref[q] + fast_log2(l_tot[q])) * kLn2 : neg_inf();
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
    wait_lds_reads();
    __bf16* orow = static_cast<__bf16*>(p.O) + row_blk * kDim;
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      const int row = ii * 8 + (lane >> 3), chunk = lane & 7;
      const u32x4 v = *reinterpret_cast<const u32x4*>(lds_kv + tile_off_bf16(row, chunk));
      *reinterpret_cast<u32x4*>(orow + row * kDim + chunk * 8) = v;
    }
#ifdef BB_STAMPS
    __builtin_amdgcn_s_waitcnt(0);
    stamp[4] = __builtin_readcyclecounter();
    if (lane == 0) {
      long long* dst = reinterpret_cast<long long*>(p.part_o) + (static_cast<size_t>(blockIdx.x) * kFwdWaves + wv) * 16;
      for (int i = 0; i < 5; ++i) dst[i] = stamp[i];
      dst[5] = cnt;
      dst[7] = stamp[5];
      dst[8] = rt0;
      dst[9] = __builtin_amdgcn_s_memrealtime();
      dst[6] = __builtin_amdgcn_s_getreg((31 << 11) | 4) /* HW_ID */;
    }
#endif
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
        pml[q * 32 + col] = m_ref[q];
        pml[kBlk + q * 32 + col] = l_tot[q];
      }
    wait_lds_reads();
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
      mrg_m[wv][q * 32 + col] = !(l_tot[q] > 0.f) ? neg_inf() : m_ref[q];
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
#ifdef BB_EXP_ONEWAVE
  hipLaunchKernelGGL(fwd_kernel_bf16, dim3(grid), dim3(kFwdThreads), 28 * 1024, stream, p);  // one workgroup per CU
#else
  hipLaunchKernelGGL(fwd_kernel_bf16, dim3(grid), dim3(kFwdThreads), 0, stream, p);
#endif
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    fprintf(stderr, "bigbird: launch of fwd_kernel_bf16 failed: %s\n", hipGetErrorString(e));
    return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
