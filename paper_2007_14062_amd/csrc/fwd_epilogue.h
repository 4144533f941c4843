// End of a forward work item: normalise and store O and LSE, or hand the partial
// (max, sum, un-normalised O) triple of a split row to the merge kernel.
#ifndef BB_FWD_EPILOGUE_H_
#define BB_FWD_EPILOGUE_H_

#include "fwd_kernels.h"

namespace bb {

// o[dt][r]: accumulator of O^T, rows d = 32*dt + acc_row(r, hf), column = query `qi`.
// m_ref: reference exponent (raw score units) the sums are relative to; l_tot: full row sum.
template <bool BF16>
__device__ __forceinline__ void fwd_store(const FwdParams& p, const WorkItem& it, const f32x16 (&o)[2],
                                          float m_ref, float l_tot, float c, size_t qrow, int qi,
                                          int hf) {
  if (it.nchunks == 1) {
    const float inv = l_tot > 0.f ? p.drop.rs / l_tot : 0.f;  // (rs: 1, or the dropout scale)
    if (hf == 0)
      p.LSE[qrow] = l_tot > 0.f ? (m_ref * c + fast_log2(l_tot)) * kLn2 : neg_inf();
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d0 = dt * 32 + acc_row(r4 * 4, hf);
        if constexpr (BF16) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[dt][r4 * 4 + e] * inv);
          *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.O) + qrow * kDim + d0) = v;
        } else {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[dt][r4 * 4 + e] * inv;
          *reinterpret_cast<f32x4*>(static_cast<float*>(p.O) + qrow * kDim + d0) = v;
        }
      }
  } else {
    float* po = p.part_o + static_cast<size_t>(it.slot) * (kBlk * kDim);
    float* pml = p.part_ml + static_cast<size_t>(it.slot) * (2 * kBlk);
    if (hf == 0) {
      pml[qi] = (m_ref == neg_inf()) ? neg_inf() : m_ref * c;
      pml[kBlk + qi] = l_tot;
    }
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d0 = dt * 32 + acc_row(r4 * 4, hf);
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = o[dt][r4 * 4 + e];
        *reinterpret_cast<f32x4*>(po + qi * kDim + d0) = v;
      }
  }
}

}  // namespace bb
#endif  // BB_FWD_EPILOGUE_H_
