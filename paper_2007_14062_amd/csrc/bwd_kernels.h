// Launch interface of the backward kernels (internal to the library).
#ifndef BB_BWD_KERNELS_H_
#define BB_BWD_KERNELS_H_

#include "dropout.h"
#include "kernel_common.h"

namespace bb {

constexpr int kMaxBwdBlocks = 256;  // longest query-block list a key block can have (LDS list): n <= 16 384,
                                    // the longest sequence the backward is verified on in full

struct BwdParams {
  const void* Q;
  const void* K;
  const void* V;
  const void* O;
  const void* dO;
  const float* LSE;
  float* dQ;
  float* dK;
  float* dV;
  const int32_t* rand_idx;
  const uint8_t* kmask;
  float* Dvec;     // [B*H*n]  -D_i, D_i = sum_c dO_ic O_ic (written by the dQ kernel)
  float* Lvec;     // [B*H*n]  LSE_i * log2(e); +inf for rows without a valid key
  float* part_dq;  // [slots][64][64] partial dQ of split rows (slots as in the forward)
  float* part_dk;  // [B*H*g*cq][64][64] partial dK of global key blocks
  float* part_dv;  // same for dV
  int B, H, BH, n, nb, g, w, r, global_mode;
  float c;      // scale * log2(e)
  float scale;
  RowSplit split;  // query-row decomposition (dQ kernel), as in the forward
  int cq;          // slices of the query-block list of a global key block: ceil(nb / 8)
  int kv_items_per_bh;  // g*cq + (nb - g)
  Dropout drop;    // attention dropout of the forward these gradients belong to (thr == 0: none)
  int skip_q;      // query blocks without a valid position (in kmask) were not computed: no gradient through them
};

// Enqueues: the dQ kernel (which also computes the row sums D), the dK/dV kernel and the
// fixed-order reductions.
int launch_bwd_bf16(const BwdParams& p, hipStream_t stream);

// The same for fp32 tensors (Q, K, V, O, dO fp32): two plain kernels, one workgroup per query
// block and per key block, no partial results (correctness configuration, not tuned).
int launch_bwd_f32(const BwdParams& p, hipStream_t stream);

}  // namespace bb
#endif  // BB_BWD_KERNELS_H_
