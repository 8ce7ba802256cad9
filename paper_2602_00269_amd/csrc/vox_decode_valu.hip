// Paged GQA decode on the vector ALU only (no matrix cores).  Kept as the measured alternative
// to the MFMA kernel; both consume the same work list and write the same partial records.
//
// One wave per (item, kv head).  Per 16-token block:
//   K granule [D/8][16][8]: lane l reads 16 bytes at (l + 64*kk)*16, i.e. token l%16 and the
//     8-dim slices l/16 + 4*kk.  Partial dot products (v_dot2_f32_bf16) of the G query heads
//     are summed over the four lane groups, so every group ends with the 16 scores.
//   online softmax per head with a 16-lane DPP max; probabilities go through a wave-private
//     LDS row so each lane can read the 8 it needs for its V slice.
//   V granule [D][16]: lane l reads 16 bytes at (l + 64*i)*16 = dim l/2 + 32*i, tokens
//     8*(l%2) .. +8; fp32 FMAs into acc[g][i]; lane pairs are summed at the end.
#include "vox_common.hpp"

namespace vox {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ inline float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// All-reduce over the 16 lanes of a DPP row: xor 1, xor 2, half mirror, mirror.
__device__ inline float row_max16(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  v = fmaxf(v, dpp_f<0x141>(v));
  v = fmaxf(v, dpp_f<0x140>(v));
  return v;
}
__device__ inline float row_sum16(float v) {
  v += dpp_f<0xB1>(v);
  v += dpp_f<0x4E>(v);
  v += dpp_f<0x141>(v);
  v += dpp_f<0x140>(v);
  return v;
}

// KV data is read once per step; non-temporal loads keep it out of the way of reused data.
__device__ inline u32x4 stream_load(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

__device__ inline float dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a),
                                         __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <int D, int G>
__global__ __launch_bounds__(256, 2) void decode_valu_kernel(
    Params p, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ bt,
    const int32_t* __restrict__ lens, const int32_t* __restrict__ header,
    const Item* __restrict__ items, float2* __restrict__ pml, float* __restrict__ pacc) {
  constexpr int NL = D / 32;  // 16-byte loads per lane per granule
  __shared__ float p_lds[kWavesPerGroup][G][kBlock];

  const int lane = threadIdx.x & (kWave - 1);
  const int wv = threadIdx.x >> 6;
  const int wid = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerGroup + wv);
  if (wid >= header[0] * p.Hkv) return;
  const int item = wid / p.Hkv, h = wid % p.Hkv;
  const Item it = items[item];
  const int s = it.stream;
  const int tok_end = min(lens[s], (it.first_block + it.nblocks) * kBlock);
  const int t = lane & 15, grp = lane >> 4, half = lane & 1;

  uint32_t qr[G][NL][4];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int kk = 0; kk < NL; ++kk) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(
          q + ((size_t)s * p.Hq + h * G + g) * D + (grp + 4 * kk) * 8);
      qr[g][kk][0] = v.x;
      qr[g][kk][1] = v.y;
      qr[g][kk][2] = v.z;
      qr[g][kk][3] = v.w;
    }

  float m[G], l[G], acc[G][NL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int i = 0; i < NL; ++i) acc[g][i] = 0.f;
  }

  const int32_t* row = bt + (size_t)s * p.max_nb + it.first_block;
  u32x4 kb[NL], vb[NL];
  {
    const size_t g0 = granule_offset(row[0], h, p.Hkv, D);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      kb[i] = stream_load(k_pool + g0 + (lane + 64 * i) * 8);
      vb[i] = stream_load(v_pool + g0 + (lane + 64 * i) * 8);
    }
  }

  for (int b = 0; b < it.nblocks; ++b) {
    u32x4 kn[NL], vn[NL];
    if (b + 1 < it.nblocks) {
      const size_t g1 = granule_offset(row[b + 1], h, p.Hkv, D);
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        kn[i] = stream_load(k_pool + g1 + (lane + 64 * i) * 8);
        vn[i] = stream_load(v_pool + g1 + (lane + 64 * i) * 8);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) kn[i] = vn[i] = u32x4{0, 0, 0, 0};
    }

    const int tok0 = (it.first_block + b) * kBlock;
    const bool valid = tok0 + t < tok_end;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float a = 0.f;
#pragma unroll
      for (int kk = 0; kk < NL; ++kk) {
        a = dot2(kb[kk].x, qr[g][kk][0], a);
        a = dot2(kb[kk].y, qr[g][kk][1], a);
        a = dot2(kb[kk].z, qr[g][kk][2], a);
        a = dot2(kb[kk].w, qr[g][kk][3], a);
      }
      a += __shfl_xor(a, 16);
      a += __shfl_xor(a, 32);
      const float sc = valid ? a * p.scale_log2 : -INFINITY;
      const float m_new = fmaxf(m[g], row_max16(sc));
      const float alpha = exp2f(m[g] - m_new);  // exp2(-inf) = 0 on the first block
      const float pr = exp2f(sc - m_new);
      l[g] = l[g] * alpha + pr;
      m[g] = m_new;
#pragma unroll
      for (int i = 0; i < NL; ++i) acc[g][i] *= alpha;
      if (grp == 0) p_lds[wv][g][t] = pr;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const bool tail = tok0 + kBlock > tok_end;  // wave-uniform
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      float v[8] = {bf16_lo(vb[i].x), bf16_hi(vb[i].x), bf16_lo(vb[i].y), bf16_hi(vb[i].y),
                    bf16_lo(vb[i].z), bf16_hi(vb[i].z), bf16_lo(vb[i].w), bf16_hi(vb[i].w)};
      if (tail) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (tok0 + half * 8 + e >= tok_end) v[e] = 0.f;  // unread slots may hold NaN
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float4 pa = *reinterpret_cast<const float4*>(&p_lds[wv][g][half * 8]);
        const float4 pb = *reinterpret_cast<const float4*>(&p_lds[wv][g][half * 8 + 4]);
        float a = acc[g][i];
        a = fmaf(pa.x, v[0], a);
        a = fmaf(pa.y, v[1], a);
        a = fmaf(pa.z, v[2], a);
        a = fmaf(pa.w, v[3], a);
        a = fmaf(pb.x, v[4], a);
        a = fmaf(pb.y, v[5], a);
        a = fmaf(pb.z, v[6], a);
        a = fmaf(pb.w, v[7], a);
        acc[g][i] = a;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      kb[i] = kn[i];
      vb[i] = vn[i];
    }
  }

#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float lsum = row_sum16(l[g]);
    const size_t rec = (size_t)item * p.Hq + h * G + g;
    if (lane == 0) pml[rec] = make_float2(m[g], lsum);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const float a = acc[g][i] + __shfl_xor(acc[g][i], 1);
      if (half == 0) pacc[rec * D + (lane >> 1) + 32 * i] = a;
    }
  }
}

template <int D>
hipError_t launch_g(const Params& p, unsigned grid, const void* q, const void* k_pool,
                    const void* v_pool, const int32_t* bt, const int32_t* lens,
                    const int32_t* header, const Item* items, float2* pml, float* pacc,
                    hipStream_t st) {
#define VOX_VALU_CASE(GG)                                                                     \
  case GG:                                                                                    \
    hipLaunchKernelGGL((decode_valu_kernel<D, GG>), dim3(grid), dim3(256), 0, st, p,          \
                       (const uint16_t*)q, (const uint16_t*)k_pool, (const uint16_t*)v_pool,  \
                       bt, lens, header, items, pml, pacc);                                   \
    break;
  switch (p.G) {
    VOX_VALU_CASE(1)
    VOX_VALU_CASE(2)
    VOX_VALU_CASE(3)
    VOX_VALU_CASE(4)
    VOX_VALU_CASE(5)
    VOX_VALU_CASE(6)
    VOX_VALU_CASE(7)
    VOX_VALU_CASE(8)
    default:
      return hipErrorInvalidValue;
  }
#undef VOX_VALU_CASE
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_valu(const Params& p, int max_wave_items, const void* q,
                              const void* k_pool, const void* v_pool, const int32_t* bt,
                              const int32_t* lens, const int32_t* header, const Item* items,
                              float2* partial_ml, float* partial_acc, hipStream_t st) {
  const unsigned grid = (unsigned)((max_wave_items + kWavesPerGroup - 1) / kWavesPerGroup);
  return p.D == 128 ? launch_g<128>(p, grid, q, k_pool, v_pool, bt, lens, header, items,
                                    partial_ml, partial_acc, st)
                    : launch_g<64>(p, grid, q, k_pool, v_pool, bt, lens, header, items,
                                   partial_ml, partial_acc, st);
}

}  // namespace vox
