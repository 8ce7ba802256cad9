// Merge of the partial (max, sum, accumulator) records of one output row: the runs of a segment
// occupy consecutive slots; lanes hold the runs' (max, sum) records, the global max and the
// rescaled sum are wave reductions, and the accumulators are combined with each lane owning
// D/64 output dims.  Used by the decode step's merge kernel.
#pragma once

#include "vox_common.hpp"

namespace vox {

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Record of run j, column col: pml[(slot0 + j) * cols + col], pacc[((slot0 + j) * cols + col) * D].
// out receives D floats (zeros when n == 0), lse one float (or is null).
template <int D>
__device__ inline void merge_runs(const float2* __restrict__ pml, const float* __restrict__ pacc,
                                  int64_t slot0, int n, int cols, int col, int lane,
                                  float* __restrict__ out, float* __restrict__ lse) {
  constexpr int DPL = D / kWave;  // dims per lane
  constexpr int kEarly = 2;       // most segments have one or two runs: their accumulators are
                                  // requested together with the (max, sum) records, not after them
  float early[kEarly][DPL];
#pragma unroll
  for (int j = 0; j < kEarly; ++j) {
    const float* src = pacc + ((size_t)(slot0 + (j < n ? j : 0)) * cols + col) * D + lane * DPL;
#pragma unroll
    for (int k = 0; k < DPL; ++k) early[j][k] = j < n ? src[k] : 0.f;
  }
  float m_run = -INFINITY, l_run = 0.f;
  float acc[DPL];
#pragma unroll
  for (int k = 0; k < DPL; ++k) acc[k] = 0.f;
  for (int c0 = 0; c0 < n; c0 += kWave) {
    const int c = c0 + lane;
    float2 ml = make_float2(-INFINITY, 0.f);
    if (c < n) ml = pml[(size_t)(slot0 + c) * cols + col];
    const float m_new = fmaxf(m_run, wave_max(ml.x));
    const float wgt = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - m_new);
    const float alpha = (m_run == -INFINITY) ? 0.f : exp2f(m_run - m_new);
    l_run = l_run * alpha + wave_sum(wgt * ml.y);
#pragma unroll
    for (int k = 0; k < DPL; ++k) acc[k] *= alpha;
    const int cnt = min(kWave, n - c0);
    int j = 0;
    if (c0 == 0) {
#pragma unroll
      for (; j < kEarly; ++j) {
        const float wj = __shfl(wgt, j);  // zero for j >= n
#pragma unroll
        for (int k = 0; k < DPL; ++k) acc[k] += wj * early[j][k];
      }
    }
    for (; j < cnt; ++j) {
      const float wj = __shfl(wgt, j);
      const float* src = pacc + ((size_t)(slot0 + c0 + j) * cols + col) * D + lane * DPL;
#pragma unroll
      for (int k = 0; k < DPL; ++k) acc[k] += wj * src[k];
    }
    m_run = m_new;
  }
  const float inv = (n > 0 && l_run > 0.f) ? 1.f / l_run : 0.f;
#pragma unroll
  for (int k = 0; k < DPL; ++k) out[lane * DPL + k] = acc[k] * inv;
  if (lse && lane == 0)
    *lse = (n > 0 && l_run > 0.f) ? (m_run + log2f(l_run)) * 0.69314718055994530942f : -INFINITY;
}

}  // namespace vox
