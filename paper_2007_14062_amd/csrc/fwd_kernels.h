// Launch interface of the forward kernels (internal to the library).
#ifndef BB_FWD_KERNELS_H_
#define BB_FWD_KERNELS_H_

#include "kernel_common.h"

namespace bb {

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
  RowSplit split;
};

// Enqueues the fused forward kernel and, if any row is split, the merge kernel.
int launch_fwd(const FwdParams& p, bool bf16, hipStream_t stream);

// The tuned bf16 main kernel (defined in fwd_bf16.hip); launch_fwd calls it.
int launch_fwd_bf16_main(const FwdParams& p, unsigned grid, hipStream_t stream);

}  // namespace bb
#endif  // BB_FWD_KERNELS_H_
