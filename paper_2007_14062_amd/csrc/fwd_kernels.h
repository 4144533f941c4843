// Launch interface of the forward kernels (internal to the library).
#ifndef BB_FWD_KERNELS_H_
#define BB_FWD_KERNELS_H_

#include "dropout.h"
#include "kernel_common.h"

namespace bb {

// Work decomposition of the bf16 forward.  Workgroups have four independent waves.
//   global workgroup: one global query block x up to 64 key blocks, 16 per wave, merged in LDS;
//   persistent workgroup: its waves take the die's other items (non-global query block x slice
//   of up to 16 key blocks: 8 at the ITC base pattern) in turn, wave w the items w, w + W, ...
// A global row longer than 64 key blocks takes several workgroups whose merged partial
// results go through the merge kernel, as do sparse rows with more than one slice.
constexpr int kGlobalWaveLen = 16;  // most key blocks a wave of a global workgroup takes
constexpr int kCounterStride = 32;  // ints between the item counters of two dies (a 128-byte line each)
struct Bf16Geom {
  int gw_len;    // key blocks per wave of a global workgroup: 16, or 8 when the whole grid fits
                 // the chip at once (then the global rows alone would set the run time)
  int ng;        // workgroups per global row: ceil(nb / (4 * gw_len))
  int cs;        // slices per non-global row: ceil(min(g + w + r, nb) / 16)
  int n_sitems;  // (nb - g) * cs
  int s_wgs;     // ceil(n_sitems / 4): workgroups the non-global items of one (batch, head) would fill
  int p_wgs;     // persistent workgroups per die: their waves share out the die's non-global items
  int g_wgs;     // global workgroups per (batch, head): g * ng
  int bh_rounds; // ceil(B*H / 8)
};

struct FwdParams {
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  float* LSE;
  const int32_t* rand_idx;
  const uint8_t* kmask;
  float* part_o;   // [slots][64][64] un-normalised partial outputs of split rows
  float* part_ml;  // [slots][2][64]  their running maxima (log2 units) and sums
  int B, H, BH, n, nb, g, w, r, global_mode;
  float c;  // scale * log2(e)
  RowSplit split;  // decomposition used by the fp32 kernel
  Bf16Geom geo;    // decomposition used by the bf16 kernel
  // rows whose slices the merge kernel combines: cmb_g_rows global rows of cmb_g_n slices each
  // (slots first), then cmb_s_rows non-global rows of cmb_s_n slices; slots_per_bh in total
  int cmb_g_rows, cmb_g_n, cmb_s_rows, cmb_s_n, slots_per_bh;
  Dropout drop;  // attention dropout (thr == 0: none)
  int skip_q;    // query blocks without a valid position (in kmask) are not computed: O = 0, LSE = -inf
  int dyn;       // bf16 kernel: waves claim their items after the first from the die's counter
  int* counters; // [8 * kCounterStride] one per die, zeroed by a small launch before the kernel (dyn != 0 only)
};

// Enqueues the fused forward kernel and, if any row is split, the merge kernel.
int launch_fwd(const FwdParams& p, bool bf16, hipStream_t stream);

// The tuned bf16 main kernel (defined in fwd_bf16.hip); launch_fwd calls it.
int launch_fwd_bf16_main(const FwdParams& p, hipStream_t stream);

}  // namespace bb
#endif  // BB_FWD_KERNELS_H_
