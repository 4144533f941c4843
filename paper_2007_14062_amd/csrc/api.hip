// C ABI entry points: host-side checks, workspace carving, kernel launches.
#include "bigbird.h"
#include "bwd_kernels.h"
#include "fwd_kernels.h"

#include <cmath>
#include <cstdio>
#include <mutex>

namespace {

constexpr size_t kAlign = 256;
inline size_t round_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WorkspaceLayout {
  size_t part_o = 0, part_ml = 0;  // forward: partial triples of split rows
  size_t counters = 0;             // forward: item counters of the dies (only if anything is carved at all)
  bool has_counters = false;
  size_t fwd_total = 0;
  // backward (its own carving of the same buffer): row sums, scaled LSE, partial gradients
  size_t dvec = 0, lvec = 0, part_dq = 0, part_dk = 0, part_dv = 0;
  size_t bwd_total = 0;
  size_t total = 0;
};

int check_attn_shape(int B, int H, int n, int d, int b, int g, int w, int r, int global_mode) {
  if (B < 0 || H < 0) return BB_ERR_SHAPE;
  int st = bb::check_pattern_args(H, n, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  if (d <= 0) return BB_ERR_SHAPE;
  if (d != bb::kDim || b != bb::kBlk) return BB_ERR_UNSUPPORTED;
  if (static_cast<long long>(B) * H > (1 << 24) || n / b > (1 << 20)) return BB_ERR_UNSUPPORTED;
  return BB_OK;
}

WorkspaceLayout make_layout(int B, int H, int n, int b, int g, int w, int r, int need_bwd) {
  WorkspaceLayout L;
  const int BH = B * H, nb = n / b;
  const bb::RowSplit s = bb::make_row_split(BH, nb, g, w, r);
  const size_t slots = static_cast<size_t>(BH) * s.slots_per_bh;
  size_t off = 0;
  L.part_o = off;
  off += round_up(slots * bb::kBlk * bb::kDim * sizeof(float));
  L.part_ml = off;
  off += round_up(slots * 2 * bb::kBlk * sizeof(float));
  if (off > 0) {
    L.counters = off;
    L.has_counters = true;
    off += round_up(bb::kXcd * bb::kCounterStride * sizeof(int));
  }
  L.fwd_total = off;
  L.total = off;
  if (need_bwd) {
    const size_t rows = static_cast<size_t>(BH) * n;
    const int cq = (nb + bb::kChunk - 1) / bb::kChunk;
    const size_t kv_slots = cq > 1 ? static_cast<size_t>(BH) * g * cq : 0;
    size_t o2 = 0;
    L.dvec = o2;
    o2 += round_up(rows * sizeof(float));
    L.lvec = o2;
    o2 += round_up(rows * sizeof(float));
    L.part_dq = o2;
    o2 += round_up(slots * bb::kBlk * bb::kDim * sizeof(float));
    L.part_dk = o2;
    o2 += round_up(kv_slots * bb::kBlk * bb::kDim * sizeof(float));
    L.part_dv = o2;
    o2 += round_up(kv_slots * bb::kBlk * bb::kDim * sizeof(float));
    L.bwd_total = o2;
    if (o2 > L.total) L.total = o2;
  }
  return L;
}

}  // namespace

extern "C" const char* bigbird_status_string(int status) {
  switch (status) {
    case BB_OK: return "ok";
    case BB_ERR_NULL: return "null pointer";
    case BB_ERR_SHAPE: return "invalid shape or pattern parameter";
    case BB_ERR_PATTERN: return "invalid random-block table";
    case BB_ERR_DTYPE: return "unknown dtype";
    case BB_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case BB_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case BB_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

extern "C" size_t bigbird_attn_workspace_bytes(int B, int H, int n, int d, int b, int g, int w,
                                               int r, int need_bwd) {
  if (check_attn_shape(B, H, n, d, b, g, w, r, BB_GLOBAL_FIRST_LAST) != BB_OK) return 0;
  return make_layout(B, H, n, b, g, w, r, need_bwd).total;
}

namespace {

const bb::Dropout kNoDropout = {0u, 0u, 0u, 1.0f};

// The forward entry points: argument checks, work decomposition, launches.  Allocates nothing.
int attn_fwd_impl(const void* Q, const void* K, const void* V, void* O, float* LSE,
                  const int32_t* rand_idx, const uint8_t* key_padding_mask, int B, int H, int n,
                  int d, int b, int g, int w, int r, float scale, int dtype, int global_mode,
                  const bb::Dropout& drop, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int skip_q = (global_mode & BB_SKIP_PADDED_QUERY_BLOCKS) != 0;
  global_mode &= ~BB_SKIP_PADDED_QUERY_BLOCKS;
  int st = check_attn_shape(B, H, n, d, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  if (dtype != BB_F32 && dtype != BB_BF16) return BB_ERR_DTYPE;
  if (!(scale > 0.f) || !std::isfinite(scale)) return BB_ERR_UNSUPPORTED;
  if (B == 0 || H == 0) return BB_OK;
  if (!Q || !K || !V || !O || !LSE) return BB_ERR_NULL;
  if (r > 0 && !rand_idx) return BB_ERR_NULL;
  const uintptr_t align_or = reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K) |
                             reinterpret_cast<uintptr_t>(V) | reinterpret_cast<uintptr_t>(O) |
                             reinterpret_cast<uintptr_t>(key_padding_mask);
  if (align_or & 15) return BB_ERR_SHAPE;
  const WorkspaceLayout L = make_layout(B, H, n, b, g, w, r, 0);
  if (L.fwd_total > 0) {
    if (!workspace || workspace_bytes < L.fwd_total ||
        (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
      return BB_ERR_WORKSPACE;
  }
  bb::FwdParams p;
  p.Q = Q; p.K = K; p.V = V; p.O = O; p.LSE = LSE;
  p.rand_idx = rand_idx;
  p.kmask = key_padding_mask;
  char* ws = static_cast<char*>(workspace);
  p.part_o = reinterpret_cast<float*>(ws + L.part_o);
  p.part_ml = reinterpret_cast<float*>(ws + L.part_ml);
  p.B = B; p.H = H; p.BH = B * H; p.n = n; p.nb = n / b;
  p.g = g; p.w = w; p.r = r; p.global_mode = global_mode;
  p.c = scale * bb::kLog2e;
  p.drop = drop;
  p.skip_q = (skip_q && key_padding_mask) ? 1 : 0;
  // When query blocks may be skipped, a fixed share of the items can be anything from all skipped
  // to all computed: the waves of the bf16 kernel then claim their items from a counter per die.
  // (Without skipped blocks claiming measured no gain over fixed shares at the key-padding
  // workload -- 60.6 against 61.1 us with its extra launch; with dropout every item is the same
  // slow path.)
  p.counters = L.has_counters ? reinterpret_cast<int*>(ws + L.counters) : nullptr;
  p.dyn = (dtype == BB_BF16 && p.skip_q && drop.thr == 0 && p.counters) ? 1 : 0;
  p.split = bb::make_row_split(p.BH, p.nb, g, w, r);
  if (dtype == BB_BF16) {
    bb::Bf16Geom& q = p.geo;
    {
      // a wave takes up to 16 key blocks of a non-global row; wider patterns are sliced
      int sparse_ub = g + w + r;
      if (sparse_ub > p.nb) sparse_ub = p.nb;
      q.cs = (sparse_ub + bb::kGlobalWaveLen - 1) / bb::kGlobalWaveLen;
      if (q.cs < 1) q.cs = 1;
    }
    q.n_sitems = (p.nb - g) * q.cs;
    q.s_wgs = (q.n_sitems + 3) / 4;
    q.bh_rounds = p.split.bh_rounds;
    // Global rows: 16 key blocks per wave (up to 64 per workgroup, merged in LDS).  When every
    // workgroup of the launch is resident at once (two per CU, 32 CUs per die) the longest
    // workgroup sets the run time, so the global rows are then cut twice as fine, into
    // workgroups whose partial results the merge kernel combines -- if that finer grid still fits.
    q.gw_len = bb::kGlobalWaveLen;
    q.ng = (p.nb + 4 * q.gw_len - 1) / (4 * q.gw_len);
    {
      const int slots_per_die = 64;
      const int fine_len = bb::kGlobalWaveLen / 2;
      const int fine_ng = (p.nb + 4 * fine_len - 1) / (4 * fine_len);
      if (p.nb > 4 * fine_len && q.bh_rounds * (g * fine_ng + q.s_wgs) <= slots_per_die) {
        q.gw_len = fine_len;
        q.ng = fine_ng;
      }
    }
    q.g_wgs = g * q.ng;
    {
      // Persistent workgroups: as many as stay resident beside the global-row workgroups (a die
      // holds 64 workgroups of this kernel: two per CU), at most one wave per item.
      const int slots_per_die = 64;
      const int n_global = q.bh_rounds * q.g_wgs;
      const int want = (q.bh_rounds * q.n_sitems + 3) / 4;
      int avail = slots_per_die - n_global;
      if (avail < 16) avail = 32;  // the global rows alone fill the die: queue behind them
      q.p_wgs = want < avail ? want : avail;
      // a wave lists the items it has to redo by the exact recurrence in one register, a lane per
      // item: no wave may be given more than 64 items, whatever that does to residency
      const int per_wave_cap = 64;
      const int floor_wgs = (q.bh_rounds * q.n_sitems + 4 * per_wave_cap - 1) / (4 * per_wave_cap);
      if (q.p_wgs < floor_wgs) q.p_wgs = floor_wgs;
    }
    p.cmb_g_rows = q.ng > 1 ? g : 0;
    p.cmb_g_n = q.ng;
    p.cmb_s_rows = q.cs > 1 ? p.nb - g : 0;
    p.cmb_s_n = q.cs;
  } else {
    p.geo = bb::Bf16Geom{};
    p.cmb_g_rows = p.split.cg > 1 ? g : 0;
    p.cmb_g_n = p.split.cg;
    p.cmb_s_rows = p.split.cs > 1 ? p.nb - g : 0;
    p.cmb_s_n = p.split.cs;
  }
  // slot numbering: the global rows' slices first, then the non-global rows' (the workspace
  // is sized for the fp32 decomposition, which never needs fewer slots)
  p.slots_per_bh = p.cmb_g_rows * p.cmb_g_n + p.cmb_s_rows * p.cmb_s_n;
  return bb::launch_fwd(p, dtype == BB_BF16, static_cast<hipStream_t>(hip_stream));
}

// Scratch memory of bigbird_attn_fwd_static: one array per GPU the library is loaded on, held
// until the process ends.  On the host the name of a __device__ array is only a handle for
// HIP_SYMBOL; the array's address on a device comes from hipGetSymbolAddress with that device
// current, once per device, and that pointer is what the kernels get.
constexpr size_t kStaticScratchBytes = BIGBIRD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // [device], nullptr until the first call on that device

int static_scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fprintf(stderr, "bigbird: bigbird_attn_fwd_static: no usable current device (%s, device %d)\n",
            hipGetErrorString(e), dev);
    return BB_ERR_LAUNCH;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fprintf(stderr, "bigbird: bigbird_attn_fwd_static: hipGetSymbolAddress failed on device %d: %s\n", dev,
              hipGetErrorString(e));
      return BB_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BB_OK;
}

}  // namespace

extern "C" int bigbird_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                int H, int n, int d, int b, int g, int w, int r, float scale,
                                int dtype, int global_mode, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  return attn_fwd_impl(Q, K, V, O, LSE, rand_idx, key_padding_mask, B, H, n, d, b, g, w, r, scale, dtype,
                       global_mode, kNoDropout, workspace, workspace_bytes, hip_stream);
}

extern "C" int bigbird_attn_fwd_dropout(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                        const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                        int H, int n, int d, int b, int g, int w, int r, float scale,
                                        int dtype, int global_mode, float p_drop, uint64_t seed,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  bb::Dropout drop;
  if (!bb::make_dropout(p_drop, seed, &drop)) return BB_ERR_SHAPE;
  return attn_fwd_impl(Q, K, V, O, LSE, rand_idx, key_padding_mask, B, H, n, d, b, g, w, r, scale, dtype,
                       global_mode, drop, workspace, workspace_bytes, hip_stream);
}

extern "C" int bigbird_dropout_keep_mask(uint8_t* keep_host, float* scale_out, float p_drop, uint64_t seed,
                                         int bh, int n, int row0, int nrows) {
  if (!keep_host) return BB_ERR_NULL;
  if (bh < 0 || n <= 0 || row0 < 0 || nrows < 0 || row0 > n - nrows) return BB_ERR_SHAPE;
  bb::Dropout drop;
  if (!bb::make_dropout(p_drop, seed, &drop)) return BB_ERR_SHAPE;
  if (scale_out) *scale_out = drop.rs;
  for (int i = 0; i < nrows; ++i) {
    const uint32_t rowid = static_cast<uint32_t>(bh) * static_cast<uint32_t>(n) + static_cast<uint32_t>(row0 + i);
    for (int j = 0; j < n; ++j)
      keep_host[static_cast<size_t>(i) * n + j] = bb::drop_keep(drop, rowid, static_cast<uint32_t>(j)) ? 1 : 0;
  }
  return BB_OK;
}

extern "C" int bigbird_attn_fwd_static(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                       const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                       int H, int n, int d, int b, int g, int w, int r, float scale,
                                       int dtype, int global_mode, void* hip_stream) {
  int st = check_attn_shape(B, H, n, d, b, g, w, r, global_mode & ~BB_SKIP_PADDED_QUERY_BLOCKS);
  if (st != BB_OK) return st;
  const size_t need = make_layout(B, H, n, b, g, w, r, 0).fwd_total;
  if (need > kStaticScratchBytes) {
    fprintf(stderr,
            "bigbird: bigbird_attn_fwd_static: these sizes need %zu bytes of scratch, the static buffer holds "
            "%zu; use bigbird_attn_fwd with a workspace of bigbird_attn_workspace_bytes()\n",
            need, kStaticScratchBytes);
    return BB_ERR_WORKSPACE;
  }
  void* ptr = nullptr;
  st = static_scratch_of_current_device(&ptr);
  if (st != BB_OK) return st;
  // Nothing in the buffer has to start at zero: every partial result a launch reads was written
  // by that launch.
  return attn_fwd_impl(Q, K, V, O, LSE, rand_idx, key_padding_mask, B, H, n, d, b, g, w, r, scale, dtype,
                       global_mode, kNoDropout, ptr, kStaticScratchBytes, hip_stream);
}

namespace {
int attn_bwd_impl(const void* Q, const void* K, const void* V, const void* O,
                  const float* LSE, const void* dO, float* dQ, float* dK, float* dV,
                  const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                  int H, int n, int d, int b, int g, int w, int r, float scale,
                  int dtype, int global_mode, const bb::Dropout& drop, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  const int skip_q = (global_mode & BB_SKIP_PADDED_QUERY_BLOCKS) != 0;
  global_mode &= ~BB_SKIP_PADDED_QUERY_BLOCKS;
  int st = check_attn_shape(B, H, n, d, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  if (dtype != BB_F32 && dtype != BB_BF16) return BB_ERR_DTYPE;
  if (!(scale > 0.f) || !std::isfinite(scale)) return BB_ERR_UNSUPPORTED;
  if (n / b > bb::kMaxBwdBlocks) return BB_ERR_UNSUPPORTED;
  if (B == 0 || H == 0) return BB_OK;
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV) return BB_ERR_NULL;
  if (r > 0 && !rand_idx) return BB_ERR_NULL;
  const uintptr_t align_or =
      reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V) |
      reinterpret_cast<uintptr_t>(O) | reinterpret_cast<uintptr_t>(dO) | reinterpret_cast<uintptr_t>(dQ) |
      reinterpret_cast<uintptr_t>(dK) | reinterpret_cast<uintptr_t>(dV) |
      reinterpret_cast<uintptr_t>(key_padding_mask);
  if (align_or & 15) return BB_ERR_SHAPE;
  const WorkspaceLayout L = make_layout(B, H, n, b, g, w, r, 1);
  if (!workspace || workspace_bytes < L.bwd_total ||
      (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
    return BB_ERR_WORKSPACE;
  bb::BwdParams p;
  p.Q = Q; p.K = K; p.V = V; p.O = O; p.dO = dO; p.LSE = LSE;
  p.dQ = dQ; p.dK = dK; p.dV = dV;
  p.rand_idx = rand_idx;
  p.kmask = key_padding_mask;
  char* ws = static_cast<char*>(workspace);
  p.Dvec = reinterpret_cast<float*>(ws + L.dvec);
  p.Lvec = reinterpret_cast<float*>(ws + L.lvec);
  p.part_dq = reinterpret_cast<float*>(ws + L.part_dq);
  p.part_dk = reinterpret_cast<float*>(ws + L.part_dk);
  p.part_dv = reinterpret_cast<float*>(ws + L.part_dv);
  p.B = B; p.H = H; p.BH = B * H; p.n = n; p.nb = n / b;
  p.g = g; p.w = w; p.r = r; p.global_mode = global_mode;
  p.c = scale * bb::kLog2e;
  p.scale = scale;
  p.drop = drop;
  p.skip_q = (skip_q && key_padding_mask) ? 1 : 0;
  p.split = bb::make_row_split(p.BH, p.nb, g, w, r);
  p.cq = (p.nb + bb::kChunk - 1) / bb::kChunk;
  p.kv_items_per_bh = g * p.cq + (p.nb - g);
  if (dtype == BB_F32) return bb::launch_bwd_f32(p, static_cast<hipStream_t>(hip_stream));
  return bb::launch_bwd_bf16(p, static_cast<hipStream_t>(hip_stream));
}
}  // namespace

extern "C" int bigbird_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                                const float* LSE, const void* dO, float* dQ, float* dK, float* dV,
                                const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                int H, int n, int d, int b, int g, int w, int r, float scale,
                                int dtype, int global_mode, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  return attn_bwd_impl(Q, K, V, O, LSE, dO, dQ, dK, dV, rand_idx, key_padding_mask, B, H, n, d, b, g, w, r,
                       scale, dtype, global_mode, kNoDropout, workspace, workspace_bytes, hip_stream);
}

extern "C" int bigbird_attn_bwd_dropout(const void* Q, const void* K, const void* V, const void* O,
                                        const float* LSE, const void* dO, float* dQ, float* dK, float* dV,
                                        const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                        int H, int n, int d, int b, int g, int w, int r, float scale,
                                        int dtype, int global_mode, float p_drop, uint64_t seed,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  bb::Dropout drop;
  if (!bb::make_dropout(p_drop, seed, &drop)) return BB_ERR_SHAPE;
  return attn_bwd_impl(Q, K, V, O, LSE, dO, dQ, dK, dV, rand_idx, key_padding_mask, B, H, n, d, b, g, w, r,
                       scale, dtype, global_mode, drop, workspace, workspace_bytes, hip_stream);
}
