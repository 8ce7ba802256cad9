// Merge of the partial (max, sum, accumulator) records of one segment (stream, kv head) by the
// wave that stored the last of them.  The runs of a segment occupy consecutive record slots;
// record x holds, for each of the G query heads of the group, (running max in log2 units, sum)
// at pml[x * G + g] and D accumulators at pacc[(x * G + g) * D].  A lane owns D/64 output dims
// of every head; runs are folded in two at a time (all loads of a pair are independent, so a
// pair costs one round trip to memory), with the usual rescaling by the running maximum.
#pragma once

#include "vox_common.hpp"

namespace vox {

// Writes out[g * D + d] for g < G (rows of the group's heads are adjacent) and lse[g].
template <int D, int G>
__device__ __forceinline__ void merge_segment_g(const float2* pml, const float* pacc, int64_t slot0, int n,
                                       int lane, float* __restrict__ out,
                                       float* __restrict__ lse) {
  constexpr int DPL = D / kWave;  // dims per lane
  float m_run[G], l_run[G], acc[G][DPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = -INFINITY;
    l_run[g] = 0.f;
#pragma unroll
    for (int k = 0; k < DPL; ++k) acc[g][k] = 0.f;
  }
  for (int j = 0; j < n; j += 2) {
    const bool two = j + 1 < n;
    const size_t ra = (size_t)(slot0 + j) * G, rb = (size_t)(slot0 + (two ? j + 1 : j)) * G;
    float2 mla[G], mlb[G];
    float a[G][DPL], b[G][DPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      mla[g] = pml[ra + g];
      mlb[g] = pml[rb + g];
#pragma unroll
      for (int k = 0; k < DPL; ++k) {
        a[g][k] = pacc[(ra + g) * D + lane * DPL + k];
        b[g][k] = pacc[(rb + g) * D + lane * DPL + k];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mb = two ? mlb[g].x : -INFINITY;
      const float m_new = fmaxf(m_run[g], fmaxf(mla[g].x, mb));
      // a record's maximum is finite (its run saw at least one token), so m_new is finite
      const float alpha = exp2f(m_run[g] - m_new);  // 0 for the first pair
      const float wa = exp2f(mla[g].x - m_new);
      const float wb = two ? exp2f(mb - m_new) : 0.f;
      l_run[g] = l_run[g] * alpha + wa * mla[g].y + wb * mlb[g].y;
#pragma unroll
      for (int k = 0; k < DPL; ++k) acc[g][k] = acc[g][k] * alpha + wa * a[g][k] + wb * b[g][k];
      m_run[g] = m_new;
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float inv = l_run[g] > 0.f ? 1.f / l_run[g] : 0.f;
#pragma unroll
    for (int k = 0; k < DPL; ++k) out[g * D + lane * DPL + k] = acc[g][k] * inv;
    if (lse && lane == 0)
      lse[g] = l_run[g] > 0.f ? (m_run[g] + log2f(l_run[g])) * 0.69314718055994530942f : -INFINITY;
  }
}

template <int D>
__device__ __forceinline__ void merge_segment(const float2* pml, const float* pacc, int64_t slot0, int n,
                                     int G, int lane, float* __restrict__ out,
                                     float* __restrict__ lse) {
  switch (G) {
    case 1: return merge_segment_g<D, 1>(pml, pacc, slot0, n, lane, out, lse);
    case 2: return merge_segment_g<D, 2>(pml, pacc, slot0, n, lane, out, lse);
    case 3: return merge_segment_g<D, 3>(pml, pacc, slot0, n, lane, out, lse);
    case 4: return merge_segment_g<D, 4>(pml, pacc, slot0, n, lane, out, lse);
    case 5: return merge_segment_g<D, 5>(pml, pacc, slot0, n, lane, out, lse);
    case 6: return merge_segment_g<D, 6>(pml, pacc, slot0, n, lane, out, lse);
    case 7: return merge_segment_g<D, 7>(pml, pacc, slot0, n, lane, out, lse);
    default: return merge_segment_g<D, 8>(pml, pacc, slot0, n, lane, out, lse);
  }
}

}  // namespace vox
