// C ABI entry points: host-side checks, workspace carving, kernel launches.
#include "bigbird.h"
#include "fwd_kernels.h"

#include <cmath>

namespace {

constexpr size_t kAlign = 256;
inline size_t round_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WorkspaceLayout {
  size_t part_o = 0, part_ml = 0;  // forward: partial triples of split rows
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
  (void)need_bwd;
  L.total = off;
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

extern "C" int bigbird_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                int H, int n, int d, int b, int g, int w, int r, float scale,
                                int dtype, int global_mode, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
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
  if (L.total > 0) {
    if (!workspace || workspace_bytes < L.total ||
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
  p.split = bb::make_row_split(p.BH, p.nb, g, w, r);
  return bb::launch_fwd(p, dtype == BB_BF16, static_cast<hipStream_t>(hip_stream));
}

extern "C" int bigbird_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                                const float* LSE, const void* dO, float* dQ, float* dK, float* dV,
                                const int32_t* rand_idx, const uint8_t* key_padding_mask, int B,
                                int H, int n, int d, int b, int g, int w, int r, float scale,
                                int dtype, int global_mode, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  (void)Q; (void)K; (void)V; (void)O; (void)LSE; (void)dO; (void)dQ; (void)dK; (void)dV;
  (void)rand_idx; (void)key_padding_mask; (void)scale; (void)dtype; (void)workspace;
  (void)workspace_bytes; (void)hip_stream;
  int st = check_attn_shape(B, H, n, d, b, g, w, r, global_mode);
  if (st != BB_OK) return st;
  return BB_ERR_UNSUPPORTED;
}
