// Block-pattern predicates shared by the host entry points and the kernels
// (App. D items 2 and 3; Sec. 2 for the ITC global set).  Integers only.
#ifndef BB_PATTERN_COMMON_H_
#define BB_PATTERN_COMMON_H_

#include "bigbird.h"

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define BB_HD __host__ __device__ __forceinline__
#else
#define BB_HD inline
#endif

namespace bb {

// The g global blocks and the clipped window of half-width (w-1)/2 on nb blocks.
struct Pattern {
  int nb;
  int g;
  int w;
  int global_mode;

  BB_HD int lead() const { return global_mode == BB_GLOBAL_LEADING ? g : (g + 1) / 2; }
  BB_HD int trail() const { return g - lead(); }
  BB_HD int half() const { return (w - 1) / 2; }
  BB_HD bool is_global(int k) const { return k < lead() || k >= nb - trail(); }
  // t-th global block, t in [0, g)
  BB_HD int global_block(int t) const { return t < lead() ? t : nb - trail() + (t - lead()); }
  // s-th non-global block, s in [0, nb - g)
  BB_HD int sparse_block(int s) const { return lead() + s; }
  // window(j) of App. D item 2, clipped to [0, nb)
  BB_HD bool in_window(int j, int k) const {
    const int dlt = k - j;
    return dlt >= -half() && dlt <= half();
  }
};

inline int check_pattern_args(int H, int n, int b, int g, int w, int r, int global_mode) {
  if (H < 0 || n <= 0 || b <= 0 || n % b != 0) return BB_ERR_SHAPE;
  if (w < 1 || (w % 2) == 0 || g < 0 || r < 0 || g > n / b) return BB_ERR_SHAPE;
  if (global_mode != BB_GLOBAL_FIRST_LAST && global_mode != BB_GLOBAL_LEADING) return BB_ERR_SHAPE;
  return BB_OK;
}

}  // namespace bb
#endif  // BB_PATTERN_COMMON_H_
