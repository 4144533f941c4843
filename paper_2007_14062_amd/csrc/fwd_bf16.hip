// bf16 forward kernel: the tuned path of the BERT-shaped workloads.
//
// Same mathematics as the fp32 kernel (eq. (AT) per head on the App. D pattern),
// organised around what limits it on this chip at d = 64: the vector port (one
// exponential per score) and the matrix pipe are within a few percent of each other,
// so every vector instruction per score counts.
//   * One wavefront owns one work item at a time: a 64-query block against a slice of
//     its key blocks (up to 16).  Waves never wait for each other inside the key-block
//     loop.  Per die, the first workgroups take one global query block each (key list
//     dealt out 16 blocks per wave, the four waves' results merged in LDS: no partial
//     results in HBM and no second kernel for up to 64 key blocks; longer rows take
//     several workgroups plus the merge kernel).  The other workgroups stay for the whole
//     launch: their waves share out the die's non-global items round robin and run them
//     as one uninterrupted stream of block pairs -- the next item's query tile and first
//     K tile ride at the end of this item's K and V tile streams, so the matrix pipe
//     only idles for the item's output.
//   * Softmax without a running maximum.  A probability is 2^(score * scale*log2(e)): one
//     multiplication and one v_exp_f32 per score, no row maximum, no accumulator rescale.
//     Softmax is shift invariant and fp32/bf16 carry eight exponent bits, so a fixed
//     reference of 0 is exact as long as the row sum stays inside [2^-40, 2^60]; a wave
//     checks that at the end of its item and, if a row left the range (logits beyond about
//     +-28 in natural units), puts the item on a list that it works off afterwards with the
//     classical running-maximum recurrence (slow_item), as it does with items that have
//     padded keys inside a block.  Both paths give the same un-normalised (reference, sum,
//     O~) triple to the common epilogue.  (Folding the factor into the query operand would
//     save the multiplication, but the operand would have to be rounded to bf16 again: that
//     perturbs a logit by up to 2^-9 of its size, four times the error of everything else in
//     LSE, and the backward pass, which recomputes the logits exactly, then sees rows whose
//     probabilities do not sum to one -- measured: gradient errors three times as large.)
//   * Row sums come from the matrix pipe as well: one small MFMA per 16 keys multiplies
//     the probabilities (already in operand layout) by a matrix of ones and zeros
//     (RowSumOperand).  That takes sixteen additions per unit off the vector port.
//   * The block pair is cut into four units (32 keys x 32 queries each) that flow through
//     a three-stage software pipeline inside the wave: scores of unit u+1 on the matrix
//     pipe, exponentials of unit u on the vector ALU, P V of unit u-1 on the matrix pipe
//     again.  The pipeline runs across key-block and item boundaries with one
//     straight-line body (pair_step) whose issue order (one MFMA, two exponentials, a
//     conversion, ...) is pinned with scheduling group barriers.  Every K and V^T operand
//     fetched from LDS feeds two MFMAs (two query tiles), which halves the LDS traffic
//     per flop.
//   * K and V tiles go global -> LDS directly (no registers in between), one 8 KB
//     buffer each, handled as 32-key halves: as soon as a half has been read out into
//     operand registers the same half of the next key block is requested, so a load has
//     three quarters of a block pair to land.
//   * V^T operands come from the transposing LDS read; the LDS layout is swizzled so
//     that neither read pattern has bank conflicts.
//   * The two waves of a SIMD get their issue priority from the pairs they still have to
//     do, so that they finish together (set_issue_priority).
//   * Two instances of the kernel.  fwd_kernel_bf16<false> is everything above and nothing else.
//     fwd_kernel_bf16<true> is launched only when a call asks for attention dropout (every item
//     then takes the per-item path, in a plain loop, where the keep mask of dropout.h is applied
//     to the probabilities that multiply V), or for fully padded query blocks to be skipped
//     (BB_SKIP_PADDED_QUERY_BLOCKS: their rows are written as zeros and the waves claim the
//     other items from a counter per die, global-row waves included once their row is done).
// -DBB_STAMPS builds a development variant that writes per-wave time stamps into the
// partial-result workspace (which must then hold 128 bytes per wave of the launch); the
// library proper is built without it.
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
__device__ __forceinline__ void half_load_async(const char* gtile_, unsigned lds, int hh,
                                                const unsigned (&voff)[2]) {
  const char* gtile = uniform_ptr(gtile_);  // wave uniform by construction: it has to sit in scalar registers
  asm volatile(
      "s_mov_b32 m0, %3\n\t"
      "s_nop 4\n\t"  // wait states the compiler cannot see to from outside: M0 written by a scalar instruction (1) and an
                       // address register pair that a vector instruction (v_readlane) may just have written (5)
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

// The lane number again, as a value the compiler cannot trace back.  Addresses and masks computed
// from it are then computed where they are used; computed from the known lane number they would
// be hoisted out of the item loop and carried through the pair loop, which has no register to
// spare (spilled, they come back one scratch load and one full memory wait at a time).
__device__ __forceinline__ int lane_again(int lane) {
  asm volatile("" : "+v"(lane));
  return lane;
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

// Issue priority of the wave by the block pairs it still has to do, in steps of four pairs: the
// two waves of a SIMD would otherwise be served oldest first, the older one would finish pairs
// ahead of the younger, and the younger would do its last pairs alone at a little more than half
// the throughput the SIMD has with two waves.  (Priority is an immediate operand.)
__device__ __forceinline__ void set_issue_priority(int remaining_pairs) {
  const int pr = remaining_pairs >> 2;
  if (pr >= 3) {
    __builtin_amdgcn_s_setprio(3);
  } else if (pr == 2) {
    __builtin_amdgcn_s_setprio(2);
  } else if (pr == 1) {
    __builtin_amdgcn_s_setprio(1);
  } else {
    __builtin_amdgcn_s_setprio(0);
  }
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
// Stage E(u): 16 exponentials, 8 conversions to bf16 pairs.
// Stage P(u): 4 MFMAs, O_q^T += V_t^T P^T, the converted scores being the B operand as they are,
//             and 2 small MFMAs for the row sums.
// Slot k of the stream issues S(k+1), E(k), P(k-1).  Unit (0,A) of the next pair is therefore
// started in the last slot of this one, and P of unit (1,B) is finished in the first slot of
// the next pair (`sA`, `p3` carry them across).
//
// Operand registers: ka[t] (K half t, "straight" fragments), va[t] (V half t, transposed
// fragments).  Each is refilled from LDS in the slot after its last use, from the half tile that
// was requested three slots earlier; the request for the half after that follows as soon as the
// read has returned.  Tile loads outstanding at the start of a pair, oldest first:
// K(i+1).t0 and V(i).t1 (8 instructions).
// Blocks with padded keys inside never come here: such items take the slow path.
struct PairCtx {
  const char* lds_k;   // this wave's K and V tile buffers
  const char* lds_v;
  unsigned lds_k_a, lds_v_a;  // the same as LDS byte addresses (scalar)
  unsigned voff[2];
  int hf;
  float c;  // scale * log2(e)
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

// Row sums on the matrix pipe.  A B operand of the 32x32x16 product (lane: query lane % 32, eight
// keys chosen by lane / 32) is read by the 16x16x32 product as column lane % 16, key group
// lane / 16: groups 0 and 2 of column c are the two key halves of query c, groups 1 and 3 those of
// query c + 16.  With an A operand whose row m is one on the groups g with m + g even and zero on
// the others, even output rows hold the sums of queries 0..15 and odd rows those of queries
// 16..31, and the output layout (lane: column lane % 16, rows 4 (lane / 16) .. + 3) gives every lane
// the total of its own query: element 0 for lane % 32 < 16, element 1 otherwise.  The sums are
// those of the rounded probabilities, the same numbers that multiply V.
struct RowSumOperand {
  bf16x8 a;
  __device__ __forceinline__ explicit RowSumOperand(int lane) {
    const __bf16 v = static_cast<__bf16>((((lane & 15) + (lane >> 4)) & 1) ? 0.f : 1.f);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = v;
  }
};
__device__ __forceinline__ float row_total(const f32x4& ls, int col) { return col < 16 ? ls[0] : ls[1]; }

// O^T += V_t^T P^T for one unit.
__device__ __forceinline__ void unit_pv(const bf16x8 (&v)[2][2], const bf16x8 (&pb)[2], f32x16 (&o)[2]) {
#pragma unroll
  for (int sgl = 0; sgl < 2; ++sgl)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v[dt][sgl], pb[sgl], o[dt], 0, 0, 0);
}

// The same, and the unit's share of the row sums.
__device__ __forceinline__ void unit_pv(const bf16x8 (&v)[2][2], const bf16x8 (&pb)[2], f32x16 (&o)[2],
                                        const RowSumOperand& ones, f32x4& ls) {
#pragma unroll
  for (int sgl = 0; sgl < 2; ++sgl) {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v[dt][sgl], pb[sgl], o[dt], 0, 0, 0);
    ls = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones.a, pb[sgl], ls, 0, 0, 0);
  }
}

// Probabilities of one unit as two B operands (16 keys each).  (The row sums are taken from these
// operands by unit_pv: sixteen additions per unit here, or eight packed bf16 dots -- which stall
// against the MFMAs in flight, measured 16 cycles each -- would sit on the vector port, which is
// the busier of the two pipes.)
__device__ __forceinline__ void unit_probs(const f32x16& s, float c, bf16x8 (&pb)[2]) {
#pragma unroll
  for (int sgl = 0; sgl < 2; ++sgl)
#pragma unroll
    for (int kk = 0; kk < 8; kk += 2) {
      const int r = sgl * 8 + kk;
      const float p0 = fast_exp2(s[r] * c);
      const float p1 = fast_exp2(s[r + 1] * c);
      const bf16x2 pk = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
      pb[sgl][kk] = pk[0];
      pb[sgl][kk + 1] = pk[1];
    }
}

// issue order of one slot: eight times (one MFMA, [LDS reads,] two exponentials), the two small
// row-sum MFMAs after the fourth and the eighth; the multiplications, conversions and lane reads
// fall where the scheduler puts them between those (pinning them too measured 1.5 % slower);
// nothing moves across the end of a slot
template <int DS_READS>
__device__ __forceinline__ void pin_slot() {
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (u * 2 < DS_READS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);  // two exponentials
    if (u == 3 || u == 7) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
}

// One block pair.  The arithmetic and the memory requests are the same for every pair, so that
// one straight-line body serves them all: the first pair of an item finishes a predecessor that
// does not exist (p3 = 0 on entry, V fragments zeroed), the last one starts a successor that does
// not exist (scores of whatever the K fragments hold, never used) -- eight idle MFMAs per item
// instead of differently scheduled copies of the body -- and a stream that has run out of tiles
// delivers a tile nobody uses (see TileStreams).
// k1 / v1: global address of the tile that follows this pair's in the K / V stream; k2: the one
// after that in the K stream.
__device__ __forceinline__ void pair_step(const PairCtx& cx, const StraightOffsets& so, const TransposedOffsets& to,
                                          const bf16x8 (&qb)[2][4], bf16x8 (&ka)[2][4], bf16x8 (&va)[2][2][2],
                                          f32x16& sA, bf16x8 (&p3)[2], f32x16 (&o)[2][2],
                                          const RowSumOperand& ones, f32x4 (&ls)[2],
                                          const char* k1, const char* v1, const char* k2) {
  f32x16 sB, sC, sD;
  bf16x8 p0[2], p1[2], p2[2];

  // ---- slot 0: the reads issued in the previous slot (K.t1, V.t0 of this pair) have returned
  wait_lds_reads();
  half_load_async(k1, cx.lds_k_a, 1, cx.voff);
  half_load_async(v1, cx.lds_v_a, 0, cx.voff);
  unit_scores(ka[0], qb[1], sB);
  unit_pv(va[1], p3, o[1], ones, ls[1]);
  unit_probs(sA, cx.c, p0);
  pin_slot<0>();

  // ---- slot 1: K(i+1).t0 and V(i).t1 have landed
  wait_tile_loads<8>();
  read_k_half(so, cx.lds_k, 0, ka[0]);
  read_v_half(to, cx.lds_v, 1, va[1]);
  unit_scores(ka[1], qb[0], sC);
  unit_pv(va[0], p0, o[0], ones, ls[0]);
  unit_probs(sB, cx.c, p1);
  pin_slot<12>();

  // ---- slot 2
  wait_lds_reads();
  half_load_async(k2, cx.lds_k_a, 0, cx.voff);
  half_load_async(v1, cx.lds_v_a, 1, cx.voff);
  unit_scores(ka[1], qb[1], sD);
  unit_pv(va[0], p1, o[1], ones, ls[1]);
  unit_probs(sC, cx.c, p2);
  pin_slot<0>();

  // ---- slot 3: K(i+1).t1 and V(i+1).t0 have landed
  wait_tile_loads<8>();
  read_k_half(so, cx.lds_k, 1, ka[1]);
  read_v_half(to, cx.lds_v, 0, va[0]);
  unit_scores(ka[0], qb[0], sA);
  unit_pv(va[1], p2, o[0], ones, ls[0]);
  unit_probs(sD, cx.c, p3);
  pin_slot<12>();
}

// LDS of a workgroup (at namespace scope: the cold paths below are separate functions).
__shared__ __attribute__((aligned(1024))) char lds_all[kFwdWaves][2 * kTile];  // per wave: K tile, V tile
__shared__ int klist_all[kFwdWaves][kGlobalWaveLen];
__shared__ float mrg_m[kFwdWaves][kBlk], mrg_l[kFwdWaves][kBlk];  // global rows: per-wave exponent, sum

// What a wave knows about itself and its LDS.
struct WaveCtx {
  int lane, wv, hf, col;
  char* lds_kv;  // this wave's 16 KB: K buffer, then V buffer
  char* lds_k;
  char* lds_v;
  int* klist;
  PairCtx cx;
  __device__ __forceinline__ explicit WaveCtx(float c) {
    lane = lane_id();
    wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, and the compiler should know
    hf = lane >> 5;
    col = lane & 31;
    lds_kv = lds_all[wv];
    lds_k = lds_kv;
    lds_v = lds_kv + kTile;
    klist = klist_all[wv];
    cx.lds_k = lds_k;
    cx.lds_v = lds_v;
    cx.hf = hf;
    cx.c = c;
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int row = par * 8 + (lane >> 3);
      cx.voff[par] = (lane >> 3) * 128 + (((lane & 7) ^ tile_swizzle(row)) << 4);
    }
    cx.lds_k_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_k));
    cx.lds_v_a = __builtin_amdgcn_readfirstlane(lds_addr(lds_v));
  }
};

// Workgroup id -> work.  id % 8 is the die (XCD) the hardware dispatches to; each die gets
// whole (batch, head) slices so that a slice's K and V stay in its L2.  The first workgroups
// of a die take one global query block each (the longest items: 16 key blocks per wave).
// The others stay for the whole launch: wave w of the die's persistent waves takes the
// non-global items w, w + wave_stride, ... of the die, in (slice, query block) order, so that
// all waves start at once and nearly all end together.
struct Sched {
  int xcd;
  unsigned wg;        // workgroup number inside the die
  unsigned n_gpart;   // global-row workgroups of the die
  bool global_wg;
  int n_items_die;    // non-global items of the die
  int wave_stride;    // persistent waves of the die
  __device__ __forceinline__ explicit Sched(const FwdParams& p) {
    xcd = blockIdx.x % kXcd;
    wg = blockIdx.x / kXcd;
    n_gpart = static_cast<unsigned>(p.geo.bh_rounds) * p.geo.g_wgs;
    global_wg = wg < n_gpart;
    const int n_bh_die = xcd < p.BH ? (p.BH - xcd + kXcd - 1) / kXcd : 0;
    n_items_die = n_bh_die * p.geo.n_sitems;
    wave_stride = p.geo.p_wgs * kFwdWaves;
  }
};

// One work item as the kernel sees it between its phases.
struct Item {
  int bh, j;           // (batch, head) slice and query block
  int chunk, nchunks;  // slice of the row's key-block list, and how many there are
  int slot;            // partial-result slot (nchunks > 1)
  int cnt;             // key blocks in this slice
  int kl;              // the list: lane t holds entry t % 16
  bool any_partial;    // some listed block has padded keys inside
  bool skipped;        // query block without a valid position, not to be computed (cnt = 0)
};

// Global addresses of an item's tiles (wave uniform, scalar arithmetic).
struct ItemTiles {
  const char* kbase;
  const char* vbase;
  const char* qtile;
  int kl;
  __device__ __forceinline__ ItemTiles(const FwdParams& p, const Item& it) {
    const size_t bh_row0 = static_cast<size_t>(it.bh) * p.n;
    kbase = static_cast<const char*>(p.K) + bh_row0 * (kDim * 2);
    vbase = static_cast<const char*>(p.V) + bh_row0 * (kDim * 2);
    qtile = static_cast<const char*>(p.Q) + (bh_row0 + it.j * kBlk) * (kDim * 2);
    kl = it.kl;
  }
  __device__ __forceinline__ const char* ktile(int i) const {
    return kbase + static_cast<size_t>(__builtin_amdgcn_readlane(kl, i)) * kTile;
  }
  __device__ __forceinline__ const char* vtile(int i) const {
    return vbase + static_cast<size_t>(__builtin_amdgcn_readlane(kl, i)) * kTile;
  }
};

// Up to four entries of a pattern-table row through the scalar data path: request and wait sit
// in one asm statement (the compiler sees the registers only once the values are in them), and
// the wait is on the scalar/LDS counter, which the tile loads in flight do not touch.
__device__ __forceinline__ void scalar_load4(const int32_t* row_, int o0, int o1, int o2, int o3, int (&e)[4]) {
  // wave uniform by construction; made so explicitly, or the operands may arrive in vector registers
  const int32_t* row = reinterpret_cast<const int32_t*>(uniform_ptr(reinterpret_cast<const char*>(row_)));
  o0 = __builtin_amdgcn_readfirstlane(o0);
  o1 = __builtin_amdgcn_readfirstlane(o1);
  o2 = __builtin_amdgcn_readfirstlane(o2);
  o3 = __builtin_amdgcn_readfirstlane(o3);
  asm volatile(
      "s_load_dword %0, %4, %5\n\t"
      "s_load_dword %1, %4, %6\n\t"
      "s_load_dword %2, %4, %7\n\t"
      "s_load_dword %3, %4, %8\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(e[0]), "=&s"(e[1]), "=&s"(e[2]), "=&s"(e[3])
      : "s"(row), "s"(o0 * 4), "s"(o1 * 4), "s"(o2 * 4), "s"(o3 * 4)
      : "memory");
}

// Does block j of batch entry bi hold a valid position?  The 64 mask bytes come through the scalar
// data path (request and wait in one statement, on the scalar counter): no vector memory wait, which
// would also wait for the tile loads in flight and for the stores of rows just written.
__device__ __forceinline__ bool block_any_valid_scalar(const uint8_t* kmask, int bi, int n, int j) {
  typedef __attribute__((ext_vector_type(16))) unsigned int u32x16;
  const char* ptr = uniform_ptr(reinterpret_cast<const char*>(kmask) + static_cast<size_t>(bi) * n + static_cast<size_t>(j) * kBlk);
  u32x16 v;
  asm volatile(
      "s_load_dwordx16 %0, %1, 0x0\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(v)
      : "s"(ptr)
      : "memory");
  unsigned any = 0;
#pragma unroll
  for (int e = 0; e < 16; ++e) any |= v[e];
  return any != 0;
}

// Item number -> item with its key-block list (for a global-row workgroup: the wave's share of
// the row).  All loads here are waited for before the function returns (scalar loads inside
// their asm statement, the others by the compiler), so tile loads in flight are at most delayed.
// Its first part: which row, which slice of the row's list (arithmetic only, no memory access).
template <bool kX>
__device__ __forceinline__ void item_coords(const FwdParams& p, const WaveCtx& w, const Sched& sc, int t, Item& it,
                                            int& list_lo, int& list_len, bool& row_global) {
  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const Bf16Geom& geo = p.geo;
  if (sc.global_wg) {
    it.bh = (sc.wg / geo.g_wgs) * kXcd + sc.xcd;
    const int gidx = sc.wg % geo.g_wgs;
    const int row = gidx / geo.ng, u = gidx % geo.ng;
    row_global = true;
    it.j = pat.global_block(row);
    it.chunk = u;
    it.nchunks = geo.ng;
    it.slot = it.bh * p.slots_per_bh + row * geo.ng + u;
    list_lo = (u * kFwdWaves + w.wv) * geo.gw_len;
    list_len = geo.gw_len;
  } else {
    // (item order inside a die: slice by slice, so that a slice's K and V stay in the L2 while its
    // rows run -- also when items are claimed: row by row across the slices, which would put the
    // rows that are not computed last, measured 52.8 against 49.2 us at the key-padding workload)
    it.bh = (t / geo.n_sitems) * kXcd + sc.xcd;
    const int sitem = t % geo.n_sitems;
    row_global = false;
    it.j = pat.sparse_block(sitem / geo.cs);
    it.chunk = sitem % geo.cs;
    it.nchunks = geo.cs;
    it.slot = it.bh * p.slots_per_bh + p.cmb_g_rows * p.cmb_g_n + sitem;
    list_lo = it.chunk * kGlobalWaveLen;  // up to 16 key blocks per item (8 at the ITC base pattern)
    list_len = kGlobalWaveLen;
  }
}

__device__ __forceinline__ const char* query_tile(const FwdParams& p, int bh, int j) {
  return static_cast<const char*>(p.Q) + (static_cast<size_t>(bh) * p.n + static_cast<size_t>(j) * kBlk) * (kDim * 2);
}

// kX (here and below): the instance of the kernel that serves attention dropout and skipped query
// blocks.  The plain instance holds none of that code, so its registers and schedule are its own.
template <bool kX>
__device__ __forceinline__ void make_item(const FwdParams& p, const WaveCtx& w, const Sched& sc, int t, Item& it) {
  const Pattern pat{p.nb, p.g, p.w, p.global_mode};
  const int lane = lane_again(w.lane);
  int list_lo, list_len;
  bool row_global;
  item_coords<kX>(p, w, sc, t, it, list_lo, list_len, row_global);
  const int bi = it.bh / p.H, h = it.bh % p.H;
  it.skipped = false;
  if (kX && p.skip_q && !block_any_valid_scalar(p.kmask, __builtin_amdgcn_readfirstlane(bi), p.n, __builtin_amdgcn_readfirstlane(it.j))) {
    // the caller reads the mask as a query mask too, and no position of this block is valid:
    // an item without key blocks (O = 0, LSE = -inf)
    it.skipped = true;
    it.any_partial = false;
    it.kl = 0;
    it.bh = __builtin_amdgcn_readfirstlane(it.bh);
    it.j = __builtin_amdgcn_readfirstlane(it.j);
    it.chunk = __builtin_amdgcn_readfirstlane(it.chunk);
    it.nchunks = __builtin_amdgcn_readfirstlane(it.nchunks);
    it.slot = __builtin_amdgcn_readfirstlane(it.slot);
    it.cnt = 0;
    return;
  }
  // Non-global rows: the table row comes through the scalar data path and the list is made
  // without a vector memory access.  A padding mask is then applied to the finished list, lane i
  // looking at block i (one round trip to memory for the whole list) -- for rows of one slice,
  // where dropping blocks afterwards cannot move a slice boundary.  Everything else takes the
  // general builder.
  const bool fast_list = !row_global && p.rand_idx && p.r > 0 &&
                         p.g + p.w + p.r <= (p.kmask ? kGlobalWaveLen : 64);
  if (fast_list) {
    const int32_t* rrow = p.rand_idx + (static_cast<size_t>(h) * p.nb + it.j) * p.r;
    int rnd = -1;
    for (int u0 = 0; u0 < p.r; u0 += 4) {
      int e[4];
      const int last = p.r - 1;
      scalar_load4(rrow, u0, u0 + 1 < last ? u0 + 1 : last, u0 + 2 < last ? u0 + 2 : last,
                   u0 + 3 < last ? u0 + 3 : last, e);
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (lane == u0 + k && u0 + k < p.r) rnd = e[k];
    }
    it.cnt = finish_key_list_sparse(pat, p.r, it.j, rnd, list_lo, list_len, w.klist);
  } else {
    it.cnt = build_key_list_range(pat, p.rand_idx, p.r, p.kmask, p.n, bi, h, it.j, row_global, list_lo,
                                  list_len, w.klist);
  }
  // same wave wrote and reads the list: LDS keeps a wave's accesses in order, the compiler must too
  asm volatile("" ::: "memory");
  it.kl = w.klist[lane & (kGlobalWaveLen - 1)];
  asm volatile("" ::: "memory");
  it.any_partial = kX && p.drop.thr != 0;  // attention dropout is applied on the slow path only
  if (p.kmask) {
    bool any_valid = false, any_padded = false;
    if (lane < it.cnt) block_mask_flags(p.kmask, bi, p.n, it.kl, any_valid, any_padded);
    if (fast_list) {
      // drop the blocks without a valid key (the general builder has done that already)
      const uint64_t m = __ballot(any_valid);
      if (any_valid) w.klist[mask_rank(m)] = it.kl;
      it.cnt = static_cast<int>(__popcll(m));
      asm volatile("" ::: "memory");
      it.kl = w.klist[lane & (kGlobalWaveLen - 1)];
      asm volatile("" ::: "memory");
    }
    it.any_partial |= __any(any_valid && any_padded) != 0;
  }
  // all of these are wave uniform; saying so keeps them (and what is computed from them) in
  // scalar registers
  it.bh = __builtin_amdgcn_readfirstlane(it.bh);
  it.j = __builtin_amdgcn_readfirstlane(it.j);
  it.chunk = __builtin_amdgcn_readfirstlane(it.chunk);
  it.nchunks = __builtin_amdgcn_readfirstlane(it.nchunks);
  it.slot = __builtin_amdgcn_readfirstlane(it.slot);
  it.cnt = __builtin_amdgcn_readfirstlane(it.cnt);
  it.any_partial = __builtin_amdgcn_readfirstlane(static_cast<int>(it.any_partial)) != 0;
}

// First tiles of an item that nobody has fetched ahead.  The query block takes the same road as a
// key block: eight coalesced 1 KB loads into LDS (the V buffer, idle until the first block's V
// arrives), then operand reads.  Register loads of the operand layout would touch every row of
// the tile in each instruction and cost the address unit four times as many cache-line requests.
// Leaves: K(0) in the K buffer, the scaled Q fragments in qb, V(0).t0 as the only load in flight.
__device__ __forceinline__ void fresh_start(const FwdParams& p, const WaveCtx& w, const StraightOffsets& so,
                                            const Item& item, bf16x8 (&qb)[2][4]) {
  const ItemTiles ct(p, item);
  tile_load_async_wave(ct.ktile(0), w.cx.lds_k_a, w.cx.voff);
  tile_load_async_wave(ct.qtile, w.cx.lds_v_a, w.cx.voff);
  wait_tile_loads<0>();
  so.read(w.lds_v, qb);
  wait_lds_reads();
  half_load_async(ct.vtile(0), w.cx.lds_v_a, 0, w.cx.voff);
}

// The two tile streams of an item as global addresses, entry m in lane m (two registers each).
// K stream: the item's K tiles; then, if an item follows, its query tile (twice: the second
// request only rewrites what the first has brought).  V stream: the item's V tiles, then the next
// item's first K tile.  So when an item's last pair is done, its successor's query tile sits in
// the K buffer and its first K tile in the V buffer (the pairs' regular reads take them for K / V
// fragments, which nothing uses).  Without a successor the streams end in the item's first tiles
// again: requests whose data nobody uses, so that every pair issues the same loads and waits for
// the same counts.
struct TileStreams {
  unsigned klo, khi, vlo, vhi;
  __device__ __forceinline__ TileStreams(const FwdParams& p, const Item& it, const Item* next, int lane) {
    const ItemTiles ct(p, it);
    // What the lanes past the item's own tiles hold.  Computed here, with every lane active: these
    // addresses read lane 0 of a list register, which must not happen inside a branch that lane 0
    // does not take (the value of an inactive lane is not defined there).
    unsigned long long k_tail, v_tail;
    if (next) {
      const ItemTiles nx(p, *next);
      k_tail = reinterpret_cast<unsigned long long>(nx.qtile);
      v_tail = reinterpret_cast<unsigned long long>(nx.ktile(0));
    } else {
      k_tail = reinterpret_cast<unsigned long long>(ct.ktile(0));
      v_tail = reinterpret_cast<unsigned long long>(ct.vtile(0));
    }
    const unsigned long long off = static_cast<unsigned long long>(static_cast<unsigned>(it.kl)) << 13;
    const bool own = lane < it.cnt;
    const unsigned long long ka = own ? reinterpret_cast<unsigned long long>(ct.kbase) + off : k_tail;
    const unsigned long long va = own ? reinterpret_cast<unsigned long long>(ct.vbase) + off : v_tail;
    klo = static_cast<unsigned>(ka);
    khi = static_cast<unsigned>(ka >> 32);
    vlo = static_cast<unsigned>(va);
    vhi = static_cast<unsigned>(va >> 32);
  }
  __device__ __forceinline__ const char* k(int m) const {
    return reinterpret_cast<const char*>(
        (static_cast<unsigned long long>(static_cast<unsigned>(__builtin_amdgcn_readlane(khi, m))) << 32) |
        static_cast<unsigned>(__builtin_amdgcn_readlane(klo, m)));
  }
  __device__ __forceinline__ const char* v(int m) const {
    return reinterpret_cast<const char*>(
        (static_cast<unsigned long long>(static_cast<unsigned>(__builtin_amdgcn_readlane(vhi, m))) << 32) |
        static_cast<unsigned>(__builtin_amdgcn_readlane(vlo, m)));
  }
};

// The item's block pairs through the pipeline.
// On entry, fresh: K(0) is in the K buffer, V(0).t0 is the only load outstanding.
//           else : K(0)'s fragments are in `ka`, V(0).t0 and V(0).t1 are outstanding, in that order
//                  (the previous item's last pairs fetched this one's first tiles, see below).
// If `nx` is given, the item after this one rides at the end of the streams: its query tile as
// one more tile of the K stream, its first K tile as one more of the V stream, so that both are
// in LDS when this item's last pair is done (they are read as K / V fragments by the pairs'
// regular reads, which nothing uses).
__device__ __forceinline__ void fast_item(const PairCtx& cx, const StraightOffsets& so, const TransposedOffsets& to,
                                          const bf16x8 (&qb)[2][4], bf16x8 (&ka)[2][4], const FwdParams& p,
                                          const Item& item, const Item* next, bool fresh,
                                          f32x16 (&o)[2][2], float (&l_tot)[2]) {
  bf16x8 va[2][2][2], p3[2];
  f32x16 sA;
  const RowSumOperand ones(lane_id());
  f32x4 ls[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};  // per query tile
#pragma unroll
  for (int a = 0; a < 2; ++a) {  // what the first pair "finishes": nothing
#pragma unroll
    for (int e = 0; e < 8; ++e) p3[a][e] = static_cast<__bf16>(0.f);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) va[1][a][b][e] = static_cast<__bf16>(0.f);
  }
  const int cnt = item.cnt;
  const TileStreams ts(p, item, next, lane_id());

  // start of the streams: K(0) -> registers, then the loads a pair expects to find outstanding
  if (fresh) {
    read_k_half(so, cx.lds_k, 0, ka[0]);
    read_k_half(so, cx.lds_k, 1, ka[1]);
    wait_lds_reads();
    half_load_async(ts.k(1), cx.lds_k_a, 0, cx.voff);
    half_load_async(ts.v(0), cx.lds_v_a, 1, cx.voff);
  } else {
    half_load_async(ts.k(1), cx.lds_k_a, 0, cx.voff);
  }
  wait_tile_loads<8>();
  read_v_half(to, cx.lds_v, 0, va[0]);
  unit_scores(ka[0], qb[0], sA);

  for (int i = 0; i < cnt; ++i)
    pair_step(cx, so, to, qb, ka, va, sA, p3, o, ones, ls, ts.k(i + 1), ts.v(i + 1), ts.k(i + 2));
  if (!next) wait_tile_loads<0>();  // requests past the end of the streams
  // the last unit's share of O and of the row sums
  unit_pv(va[1], p3, o[1], ones, ls[1]);
#pragma unroll
  for (int q = 0; q < 2; ++q) l_tot[q] = row_total(ls[q], lane_id() & 31);
}

// The classical recurrence (running maximum, rescale on every block), one block pair at a time
// with synchronous tile loads: the path of items with padded keys inside a block and the
// fallback for items whose row sums left the safe range of the reference-free path.  Leaves m_ref (exponent
// units), this lane's share of the row sums and O~.  Any load still in flight lands first.
template <bool kX>
__device__ __forceinline__ void slow_item(const PairCtx& cx, const StraightOffsets& so, const TransposedOffsets& to,
                                          const bf16x8 (&qb)[2][4], const FwdParams& p, const Item& item,
                                          f32x16 (&o)[2][2], float (&l_run)[2], float (&m_ref)[2]) {
  const ItemTiles it(p, item);
  zero_acc(o[0]);
  zero_acc(o[1]);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    m_ref[q] = neg_inf();
    l_run[q] = 0.f;
  }
  // attention dropout (all items of a call with dropout come here): the keys of this lane's two
  // rows of the keep mask
  uint32_t drop_rk[2] = {0u, 0u};
  if (kX && p.drop.thr) {
    const uint32_t row0 = static_cast<uint32_t>(item.bh) * static_cast<uint32_t>(p.n) + item.j * kBlk + (lane_id() & 31);
#pragma unroll
    for (int q = 0; q < 2; ++q) drop_rk[q] = drop_row_key(p.drop, row0 + q * 32);
  }
  // The tiles of pair i + 1 are requested as soon as those of pair i sit in registers, and land
  // under pair i's arithmetic.
  auto request_tiles = [&](int i) {
    const char* kt = it.ktile(i);
    const char* vt = it.vtile(i);
    half_load_async(kt, cx.lds_k_a, 0, cx.voff);
    half_load_async(kt, cx.lds_k_a, 1, cx.voff);
    half_load_async(vt, cx.lds_v_a, 0, cx.voff);
    half_load_async(vt, cx.lds_v_a, 1, cx.voff);
  };
  if (item.cnt > 0) request_tiles(0);
  for (int i = 0; i < item.cnt; ++i) {
    const int kblock = __builtin_amdgcn_readlane(item.kl, i);
    uint64_t vbits = ~0ull;
    if (p.kmask) vbits = key_valid_bits(p.kmask, item.bh / p.H, p.n, kblock);
    wait_tile_loads<0>();
    bf16x8 ka[2][4], va[2][2][2];
    read_k_half(so, cx.lds_k, 0, ka[0]);
    read_k_half(so, cx.lds_k, 1, ka[1]);
    read_v_half(to, cx.lds_v, 0, va[0]);
    read_v_half(to, cx.lds_v, 1, va[1]);
    wait_lds_reads();  // the buffers are free again
    if (i + 1 < item.cnt) request_tiles(i + 1);
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
          s[t][r] = ((mine >> acc_row(r, 0)) & 1) ? s[t][r] * cx.c : neg_inf();  // base-2 exponent
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
            const float p0 = fast_exp2(s[t][r] - m_use), p1 = fast_exp2(s[t][r + 1] - m_use);
            bf16x2 pk = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
            l_run[q] += p0 + p1;  // (the row sums are those of the undropped probabilities)
            if (kX && p.drop.thr) {
              // registers r, r + 1 are keys 2m, 2m + 1: one word of the mask
              const uint32_t key = static_cast<uint32_t>(kblock * kBlk + t * 32 + acc_row(r, cx.hf));
              const uint32_t wd = drop_word(drop_rk[q], key >> 1);
              if (!drop_keep_even(wd, p.drop.thr)) pk[0] = static_cast<__bf16>(0.f);
              if (!drop_keep_odd(wd, p.drop.thr)) pk[1] = static_cast<__bf16>(0.f);
            }
            pb[sgl][kk] = pk[0];
            pb[sgl][kk + 1] = pk[1];
          }
        unit_pv(va[t], pb, o[q]);
      }
    }
  }
}

// Normalised bf16 output and LSE of a non-global item.  The accumulators hold O^T (a lane owns one
// query and scattered groups of four d); they are turned through LDS (the K buffer) so that global
// memory sees whole rows: 16 bytes per lane, consecutive lanes on consecutive addresses.
__device__ __forceinline__ void store_rows_bf16(const FwdParams& p, const WaveCtx& w, const Item& it,
                                                const f32x16 (&o)[2][2], const float (&inv)[2],
                                                const float (&lse)[2]) {
  const size_t row_blk = static_cast<size_t>(it.bh) * p.n + it.j * kBlk;  // first row of the query block
  const int lane = lane_again(w.lane), hf = lane >> 5, col = lane & 31;
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (hf == 0) p.LSE[row_blk + q * 32 + col] = lse[q];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[q][dt][r4 * 4 + e] * inv[q]);
        // d0 = 32 dt + 8 r4 + 4 hf: 16-byte chunk 4 dt + r4, upper or lower half of it
        *reinterpret_cast<bf16x4*>(w.lds_k + tile_off_bf16(q * 32 + col, dt * 4 + r4) + hf * 8) = v;
      }
  }
  wait_lds_reads();
  __bf16* orow = static_cast<__bf16*>(p.O) + row_blk * kDim;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    u32x4 ov[4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
      ov[ii] = *reinterpret_cast<const u32x4*>(w.lds_k +
                                               tile_off_bf16((half * 4 + ii) * 8 + (lane >> 3), lane & 7));
    wait_lds_reads();  // after the second batch the K buffer may be refilled
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
      // (non-temporal: the output is not read again, and K and V need the L2: 0.5 us at cfg 2)
      __builtin_nontemporal_store(ov[ii], reinterpret_cast<u32x4*>(orow + ((half * 4 + ii) * 8 + (lane >> 3)) * kDim + (lane & 7) * 8));
  }
}

// Partial triple (reference exponent, row sums, un-normalised O in fp32) of one slice of a row
// that has several, for the merge kernel; O goes through the K buffer in two passes of 32 d.
__device__ __forceinline__ void store_partial(const FwdParams& p, const WaveCtx& w, const Item& it,
                                              const f32x16 (&o)[2][2], const float (&m_ref)[2],
                                              const float (&l_tot)[2]) {
  const int lane = lane_again(w.lane), hf = lane >> 5, col = lane & 31;
  float* pml = p.part_ml + static_cast<size_t>(it.slot) * (2 * kBlk);
  float* po = p.part_o + static_cast<size_t>(it.slot) * (kBlk * kDim);
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (hf == 0) {
      pml[q * 32 + col] = m_ref[q];
      pml[kBlk + q * 32 + col] = l_tot[q];
    }
#pragma unroll
  for (int dt = 0; dt < 2; ++dt) {
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = o[q][dt][r4 * 4 + e];
        *reinterpret_cast<f32x4*>(w.lds_k + tile_off_bf16(q * 32 + col, r4 * 2 + hf)) = v;
      }
    wait_lds_reads();
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      const int row = ii * 8 + (lane >> 3), cc = lane & 7;
      const f32x4 v = *reinterpret_cast<const f32x4*>(w.lds_k + tile_off_bf16(row, cc));
      *reinterpret_cast<f32x4*>(po + row * kDim + dt * 32 + cc * 4) = v;
    }
    wait_lds_reads();
  }
}

// O = 0 and LSE = -inf for the 64 rows of a query block that is not computed (whole rows, 16 bytes
// per lane, straight from registers).
__device__ __forceinline__ void store_zero_rows_bf16(const FwdParams& p, const Item& it) {
  const size_t row_blk = static_cast<size_t>(it.bh) * p.n + it.j * kBlk;
  const int lane = lane_id();
  p.LSE[row_blk + lane] = neg_inf();
  __bf16* orow = static_cast<__bf16*>(p.O) + row_blk * kDim;
  const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int ii = 0; ii < 8; ++ii)
    __builtin_nontemporal_store(z, reinterpret_cast<u32x4*>(orow + (ii * 8 + (lane >> 3)) * kDim + (lane & 7) * 8));
}

// The kernel's argument block as the cold functions below see it.  A reference to the kernel's own
// copy would move that copy, and every later use of it in the hot loop, into scratch memory, and the
// kernel-argument segment pointer is only defined inside the kernel itself.  So the kernel hands its
// segment pointer down and the callee reads the structure again through scalar loads.
typedef const FwdParams __attribute__((address_space(4))) * KernargPtr;

__device__ __forceinline__ FwdParams params_from(const void* kernargs) {
#if defined(__HIP_DEVICE_COMPILE__)
  const char* u = uniform_ptr(static_cast<const char*>(kernargs));
  return *(KernargPtr)(reinterpret_cast<uintptr_t>(u));
#else
  return FwdParams{};
#endif
}

__device__ __forceinline__ const void* kernel_kernargs() {
#if defined(__HIP_DEVICE_COMPILE__)
  return (const void*)(__builtin_amdgcn_kernarg_segment_ptr());
#else
  return nullptr;
#endif
}

// One non-global item by the classical recurrence, from its first load to its last store: the path
// of items with padded keys inside a block or without any key block, and of items whose row sums
// left the safe range of the pipelined path, and of every item under attention dropout.
template <bool kX>
__device__ __forceinline__ void item_by_recurrence(const FwdParams& p, int t) {
  const WaveCtx w(p.c);
  Sched sc(p);
  sc.global_wg = false;  // (a wave of a global-row workgroup that went on to claim other items)
  const StraightOffsets so(w.lane);
  const TransposedOffsets to(w.lane);
  Item it;
  make_item<kX>(p, w, sc, t, it);
  wait_tile_loads<0>();
  bf16x8 qb[2][4];
  f32x16 o[2][2];
  float l_run[2], m_ref[2], l_tot[2];
  if (it.cnt > 0) {
    tile_load_async_wave(ItemTiles(p, it).qtile, w.cx.lds_v_a, w.cx.voff);
    wait_tile_loads<0>();
    so.read(w.lds_v, qb);
    wait_lds_reads();
    }
  slow_item<kX>(w.cx, so, to, qb, p, it, o, l_run, m_ref);
#pragma unroll
  for (int q = 0; q < 2; ++q) l_tot[q] = half_sum(l_run[q]);
  if (it.nchunks == 1) {
    float inv[2], lse[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      inv[q] = l_tot[q] > 0.f ? (kX ? p.drop.rs : 1.f) / l_tot[q] : 0.f;  // (rs: 1, or the dropout scale)
      lse[q] = l_tot[q] > 0.f ? (m_ref[q] + fast_log2(l_tot[q])) * kLn2 : neg_inf();
    }
    store_rows_bf16(p, w, it, o, inv, lse);
  } else {
    store_partial(p, w, it, o, m_ref, l_tot);
  }
}

// The persistent loop's list of such items (lane u of `redo` holds the u-th item), as a called
// function: its registers are not that loop's problem.  One call for the whole list: a call saves
// and restores the callee-saved registers in scratch memory, about 50 KB per wave, which per item
// was most of the time of launches in which many items come here.
template <bool kX>
__device__ __attribute__((noinline)) void redo_items(const void* kernargs, int redo, int n_redo) {
  const FwdParams p = params_from(kernargs);
  for (int u = 0; u < n_redo; ++u) item_by_recurrence<kX>(p, __builtin_amdgcn_readlane(redo, u));
}

// One global query block by a whole workgroup: 16 key blocks per wave, the four waves' (m, l, O~)
// merged in LDS.  Inlined into the kernel, as the branch taken by the die's first workgroups: a
// real call would start by saving a hundred callee-saved vector registers to scratch memory
// (11 MB of HBM writes per launch at the BERT-base size, measured) for a caller that has nothing
// in them.
template <bool kX>
__device__ __forceinline__ void global_row_workgroup(const FwdParams& p) {
  const WaveCtx w(p.c);
  const Sched sc(p);
  const StraightOffsets so(w.lane);
  const TransposedOffsets to(w.lane);
  const int lane = w.lane, wv = w.wv, hf = w.hf, col = w.col;
#ifdef BB_STAMPS
  const long long rt0 = __builtin_amdgcn_s_memrealtime();
#endif
  Item cur;
  make_item<kX>(p, w, sc, 0, cur);
  bf16x8 qb[2][4], ka[2][4];
  f32x16 o[2][2];
  float m_ref[2] = {0.f, 0.f};  // reference exponents (base-2 units); halves agree
  float l_tot[2] = {0.f, 0.f};  // row sums of 2^(s - m_ref)
  zero_acc(o[0]);
  zero_acc(o[1]);
  if (cur.cnt > 0) {
    fresh_start(p, w, so, cur, qb);
    float l_run[2] = {0.f, 0.f};
    bool bad = cur.any_partial;  // per-key masking is only in the slow path
    if (!cur.any_partial) {
      fast_item(w.cx, so, to, qb, ka, p, cur, nullptr, true, o, l_tot);
#pragma unroll
      for (int q = 0; q < 2; ++q) bad |= !(l_tot[q] >= kSumLo && l_tot[q] <= kSumHi);
    }
    if (__any(bad)) {
      slow_item<kX>(w.cx, so, to, qb, p, cur, o, l_run, m_ref);
#pragma unroll
      for (int q = 0; q < 2; ++q) l_tot[q] = half_sum(l_run[q]);
    }
  } else {
    m_ref[0] = m_ref[1] = neg_inf();
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
        *reinterpret_cast<f32x4*>(w.lds_kv + dt * kTile + tile_off_bf16(q * 32 + col, r4 * 2 + hf)) = v;
      }
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (hf == 0) {
      mrg_m[wv][q * 32 + col] = !(l_tot[q] > 0.f) ? neg_inf() : m_ref[q];
      mrg_l[wv][q * 32 + col] = l_tot[q];
    }
#ifdef BB_STAMPS
  if (lane == 0) {  // (nchunks == 1 only: the partial-result area is otherwise in use)
    long long* dst = reinterpret_cast<long long*>(p.part_o) + (static_cast<size_t>(blockIdx.x) * kFwdWaves + wv) * 16;
    dst[0] = rt0;
    dst[1] = __builtin_amdgcn_s_memrealtime();
    dst[2] = -1;
    dst[15] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | (31 << 11));  // HW_ID: where the wave ran
  }
#endif
  __syncthreads();  // all four waves of a global workgroup arrive here
  // wave w now owns query rows 16w .. 16w+15; a lane owns 16 d columns of one row
  const size_t row_blk = static_cast<size_t>(cur.bh) * p.n + cur.j * kBlk;
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
        const f32x4 x = *reinterpret_cast<const f32x4*>(lds_all[v] + (cc >> 3) * kTile + tile_off_bf16(q, cc & 7));
#pragma unroll
        for (int z = 0; z < 4; ++z) acc[e][z] += x[z] * wgt;
      }
    }
  }
  const size_t row = row_blk + q;
  if (cur.nchunks == 1) {
    const float inv = L > 0.f ? (kX ? p.drop.rs : 1.f) / L : 0.f;  // (rs: 1, or the dropout scale)
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
    float* pml = p.part_ml + static_cast<size_t>(cur.slot) * (2 * kBlk);
    if (part == 0) {
      pml[q] = L > 0.f ? M : neg_inf();
      pml[kBlk + q] = L;
    }
    f32x4* dst =
        reinterpret_cast<f32x4*>(p.part_o + static_cast<size_t>(cur.slot) * (kBlk * kDim) + q * kDim + part * 16);
#pragma unroll
    for (int e = 0; e < 4; ++e) dst[e] = acc[e];
  }
}

}  // namespace

// The item counters of the dies start every launch at zero (a kernel, not a memset: the call may
// be under graph capture).
__global__ void zero_counters_kernel(int* counters) {
  if (threadIdx.x < kXcd) counters[threadIdx.x * kCounterStride] = 0;
}

template <bool kX>
__global__ __launch_bounds__(kFwdThreads) __attribute__((amdgpu_waves_per_eu(2)))
void fwd_kernel_bf16(FwdParams p) {
  Sched sc(p);
  // dyn: after its first piece of work a wave claims items from its die's counter (zeroed before
  // the launch) instead of taking every wave_stride-th one: with a padding mask items differ in
  // length and some are not computed at all.  The waves of a global-row workgroup then join in
  // when their row is done.
  const bool dyn = kX && p.dyn != 0;
  const bool was_global = sc.global_wg;
  if (sc.global_wg) {
    if ((sc.wg / p.geo.g_wgs) * kXcd + sc.xcd < static_cast<unsigned>(p.BH)) global_row_workgroup<kX>(p);
    if (!dyn) return;
    __syncthreads();  // the merge has read the other waves' LDS regions; from here on each wave's is its own
    sc.global_wg = false;
  }
  const WaveCtx w(p.c);
  const PairCtx& cx = w.cx;
  const int lane = w.lane;
  char* const lds_k = w.lds_k;
  char* const lds_v = w.lds_v;
  const StraightOffsets so(lane);
  const TransposedOffsets to(lane);
  const int n_items_die = sc.n_items_die, wave_stride = sc.wave_stride;
  // the die's next unclaimed item (tickets start after the items the persistent waves begin with)
  auto claim = [&]() {
    int c = 0;
    // Executed in the die's L2, which all claimers of this counter share (a counter per die, a
    // cache line each).  Were two dies ever to work on one counter, each would see its own copy:
    // items done twice with the same result, none left out.
    if (lane == 0)
      c = __hip_atomic_fetch_add(p.counters + sc.xcd * kCounterStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    c = __builtin_amdgcn_readfirstlane(c);
    // (a counter that has run far past the end must not wrap the sum)
    return c < n_items_die ? wave_stride + c : n_items_die;
  };
  if (kX && p.drop.thr != 0) {
    // attention dropout: every item takes the per-item path, so there is no stream to run and no
    // list to keep -- wave w does the die's items w, w + wave_stride, ... one after the other
    for (int t = static_cast<int>(sc.wg - sc.n_gpart) * kFwdWaves + w.wv; t < n_items_die; t += wave_stride)
      item_by_recurrence<kX>(p, __builtin_amdgcn_readfirstlane(t));
    return;
  }
  int t_first = static_cast<int>(sc.wg - sc.n_gpart) * kFwdWaves + w.wv;  // first item of this wave
  if (dyn && was_global) t_first = claim();
  const int t_item = __builtin_amdgcn_readfirstlane(t_first);
  if (t_item >= n_items_die) return;

  bf16x8 qb[2][4];  // Q^T operands (B of S^T = K Q^T): lane holds query `col` (+32 for tile B),
                    // d = 16*ks + 8*hf .. +8 -- the "straight" fragments of the Q tile, scaled
  bf16x8 ka[2][4];  // K fragments of the pair in work (they cross the item boundary)
  f32x16 o[2][2];   // [query tile][d tile]: O^T accumulators

#ifdef BB_STAMPS
  // development build (-DBB_STAMPS): per-wave time accounting into the partial-result workspace,
  // 16 x 8 bytes per wave: start and end on the constant 100 MHz clock, items done, shader-clock
  // sums per phase of the persistent loop
  const long long rt0 = __builtin_amdgcn_s_memrealtime();
  long long acc_t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  long long st_t[4] = {0, 0, 0, 0};  // first start in detail: lists, first tiles, operands ready
  long long tprev = __builtin_readcyclecounter();
  int n_done = 0;
#define BB_STAMP(i) do { const long long tn__ = __builtin_readcyclecounter(); acc_t[i] += tn__ - tprev; tprev = tn__; } while (0)
#else
#define BB_STAMP(i)
#endif
  // ---- persistent wave: the die's non-global items t_item, t_item + wave_stride, ...
  // Items that cannot take the pipelined path (padded keys inside a block, no key block at all,
  // or -- found out afterwards -- row sums outside the safe range) are put on a list and done
  // by the classical recurrence when the stream has ended; the host sizes the grid so that a
  // wave has at most 64 items (a lane of `redo` each).
  int redo = 0;       // the list: lane t holds the number of the t-th such item
  int n_redo = 0;
  auto push_redo = [&](int t) {
    if (lane == n_redo) redo = t;
    n_redo = __builtin_amdgcn_readfirstlane(n_redo + 1);
  };
  // the next item at or after t that takes the pipelined path (others go to the list)
  auto next_fast = [&](int t, Item& it) {
    int found = -1;
    while (t < n_items_die) {
      make_item<kX>(p, w, sc, t, it);
      if (it.cnt > 0 && !it.any_partial) {
        found = t;
        break;
      }
      if (kX && it.skipped && it.nchunks == 1) {  // nothing to compute: its rows are written here
        store_zero_rows_bf16(p, it);
      } else {
        push_redo(t);
      }
      if (dyn) {
        if (n_redo >= 64) break;  // the list is full: this wave takes no more items, the others do
        t = claim();
      } else {
        t += wave_stride;
      }
    }
    return __builtin_amdgcn_readfirstlane(found);
  };
  // where the search for the item after item t begins
  auto successor = [&](int t) { return dyn ? (n_redo < 64 ? claim() : n_items_die) : t + wave_stride; };

  // cur: the item in work; nxt: the one after it (its list is needed before cur's last pairs,
  // which fetch its first tiles); nn: the one after that, built while few loads are in flight.
  // Where the first item's row is does not depend on the pattern table: its query tile is
  // requested (into the K buffer) before anything else, and the table is read under that flight.
  Item cur, nxt, nn;
  {
    int lo_, len_;
    bool rg_;
    item_coords<kX>(p, w, sc, t_item, cur, lo_, len_, rg_);
    tile_load_async_wave(query_tile(p, __builtin_amdgcn_readfirstlane(cur.bh), __builtin_amdgcn_readfirstlane(cur.j)),
                         cx.lds_k_a, cx.voff);
  }
  int t_cur = next_fast(t_item, cur);
  int t_nxt = -1;
#ifdef BB_STAMPS
  st_t[0] = __builtin_readcyclecounter() - tprev;
#endif
  if (t_cur < 0) wait_tile_loads<0>();  // nothing for the pipelined path: let the request land
  if (t_cur >= 0) {
    bf16x8 va[2][2][2], p3[2];
    f32x16 sA;
    const RowSumOperand ones(lane_again(lane));
    f32x4 ls[2];
    // what the first pair of an item "finishes": nothing
    auto reset_item_state = [&]() {
      zero_acc(o[0]);
      zero_acc(o[1]);
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        ls[a] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 8; ++e) p3[a][e] = static_cast<__bf16>(0.f);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int e = 0; e < 8; ++e) va[1][a][b][e] = static_cast<__bf16>(0.f);
      }
    };
    // pairs this wave still has to do, roughly (for its issue priority)
    const int pairs_per_item = p.geo.cs > 1 ? kGlobalWaveLen : (p.g + p.w + p.r < kGlobalWaveLen ? p.g + p.w + p.r : kGlobalWaveLen);
    int rem_pairs = dyn ? 0  // (unknown when items are claimed: every wave at the same priority)
                        : __builtin_amdgcn_readfirstlane(((n_items_die - t_cur + wave_stride - 1) / wave_stride) * pairs_per_item);

    // start of the first item.  Skipped items ahead of it: the request above was for another row.
    wait_tile_loads<0>();
    if (t_cur != t_item) {
      tile_load_async_wave(query_tile(p, cur.bh, cur.j), cx.lds_k_a, cx.voff);
      wait_tile_loads<0>();
    }
    so.read(lds_k, qb);
    wait_lds_reads();
    {
      // K(0) and V(0) together; the next item's list is made while they fly
      const ItemTiles ct(p, cur);
      tile_load_async_wave(ct.ktile(0), cx.lds_k_a, cx.voff);
      const char* v0 = uniform_ptr(ct.vtile(0));
      half_load_async(v0, cx.lds_v_a, 0, cx.voff);
      half_load_async(v0, cx.lds_v_a, 1, cx.voff);
    }
#ifdef BB_STAMPS
    st_t[2] = __builtin_readcyclecounter() - tprev;
#endif
    t_nxt = next_fast(successor(t_cur), nxt);  // (scalar loads only, unless there is a padding mask)
    TileStreams ts(p, cur, t_nxt >= 0 ? &nxt : nullptr, lane_again(lane));
    int cnt = __builtin_amdgcn_readfirstlane(cur.cnt);  // pairs of the item in work
      reset_item_state();
#ifdef BB_STAMPS
    st_t[1] = __builtin_readcyclecounter() - tprev;
#endif
    wait_tile_loads<8>();  // K(0)
    read_k_half(so, lds_k, 0, ka[0]);
    read_k_half(so, lds_k, 1, ka[1]);
    wait_lds_reads();
    half_load_async(ts.k(1), cx.lds_k_a, 0, cx.voff);
    wait_tile_loads<8>();  // V(0).t0
    read_v_half(to, lds_v, 0, va[0]);
    unit_scores(ka[0], qb[0], sA);
    BB_STAMP(0);

    for (int i = 0;;) {
      if ((rem_pairs & 3) == 3 || i == 0) set_issue_priority(rem_pairs);
      pair_step(cx, so, to, qb, ka, va, sA, p3, o, ones, ls, ts.k(i + 1), ts.v(i + 1), ts.k(i + 2));
      rem_pairs = __builtin_amdgcn_readfirstlane(rem_pairs - 1);
      i = __builtin_amdgcn_readfirstlane(i + 1);
      if (__builtin_expect(i < cnt, 1)) continue;  // (the register allocator should favour the pairs)

      // ---- item boundary.  The last unit's share of O, the row sums, the range check.
      BB_STAMP(1);
      unit_pv(va[1], p3, o[1], ones, ls[1]);
      bool bad = false;
      float inv[2], lse[2], lsum[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const float l = row_total(ls[q], w.col);
        bad |= !(l >= kSumLo && l <= kSumHi);
        lsum[q] = l;
        inv[q] = 1.f / l;
        lse[q] = fast_log2(l) * kLn2;
      }
      const bool redo_cur = __any(bad);
      if (redo_cur) push_redo(t_cur);

      // the list of the item after the next: here at most four tile loads are in flight, so the
      // waits that building it may need (compiler-placed, for all loads) cost little
      int t_nn = -1;
      BB_STAMP(2);
      if (t_nxt >= 0) {
        t_nn = next_fast(successor(t_nxt), nn);
        BB_STAMP(3);
        // The next item's query tile is in the K buffer, its first K tile in the V buffer (the
        // second half may still be landing).  Both go to registers, its first V tile is requested,
        // and this item's output is written under that flight.
        wait_tile_loads<0>();
        so.read(lds_k, qb);
        read_k_half(so, lds_v, 0, ka[0]);
        read_k_half(so, lds_v, 1, ka[1]);
        wait_lds_reads();
        const char* v0 = uniform_ptr(ItemTiles(p, nxt).vtile(0));
        half_load_async(v0, cx.lds_v_a, 0, cx.voff);
        half_load_async(v0, cx.lds_v_a, 1, cx.voff);
      }

      BB_STAMP(4);
      if (t_nxt < 0) wait_tile_loads<0>();  // requests past the end of the streams
      // ---- output, through the K buffer (free now)
      if (!redo_cur) {
        if (cur.nchunks == 1) {
          store_rows_bf16(p, w, cur, o, inv, lse);
        } else {
          const float zero[2] = {0.f, 0.f};
          store_partial(p, w, cur, o, zero, lsum);
        }
      }
      BB_STAMP(5);
#ifdef BB_STAMPS
      ++n_done;
#endif
      if (t_nxt < 0) break;

      // ---- the next item's stream starts (its K(0) fragments are in registers, V(0) is in flight)
          cur = nxt;
      t_cur = t_nxt;
      nxt = nn;
      t_nxt = t_nn;
      ts = TileStreams(p, cur, t_nxt >= 0 ? &nxt : nullptr, lane_again(lane));
      reset_item_state();
      cnt = __builtin_amdgcn_readfirstlane(cur.cnt);
      half_load_async(ts.k(1), cx.lds_k_a, 0, cx.voff);
      wait_tile_loads<8>();
      read_v_half(to, lds_v, 0, va[0]);
      unit_scores(ka[0], qb[0], sA);
      i = 0;
      BB_STAMP(6);
    }
  }
#ifdef BB_STAMPS
  if (lane == 0) {
    long long* dst = reinterpret_cast<long long*>(p.part_o) + (static_cast<size_t>(blockIdx.x) * kFwdWaves + w.wv) * 16;
    dst[0] = rt0;
    dst[1] = __builtin_amdgcn_s_memrealtime();
    dst[2] = n_done;
    for (int i = 0; i < 7; ++i) dst[3 + i] = acc_t[i];
    dst[10] = st_t[0];
    dst[11] = st_t[1];
    dst[12] = st_t[2];
    dst[15] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | (31 << 11));  // HW_ID: where the wave ran
  }
#endif

  // ---- the listed items, by the classical recurrence
  if (n_redo > 0) redo_items<kX>(kernel_kernargs(), redo, n_redo);
}

int launch_fwd_bf16_main(const FwdParams& p, hipStream_t stream) {
  const unsigned grid = static_cast<unsigned>(kXcd) * (p.geo.bh_rounds * p.geo.g_wgs + p.geo.p_wgs);
  if (grid == 0) return BB_OK;
  if (p.dyn) {
    hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, stream, p.counters);
    if (hipGetLastError() != hipSuccess) return BB_ERR_LAUNCH;
  }
  if (p.drop.thr != 0 || p.skip_q || p.dyn)
    hipLaunchKernelGGL(fwd_kernel_bf16<true>, dim3(grid), dim3(kFwdThreads), 0, stream, p);
  else
    hipLaunchKernelGGL(fwd_kernel_bf16<false>, dim3(grid), dim3(kFwdThreads), 0, stream, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    fprintf(stderr, "bigbird: launch of fwd_kernel_bf16 failed: %s\n", hipGetErrorString(e));
    return BB_ERR_LAUNCH;
  }
  return BB_OK;
}

}  // namespace bb
