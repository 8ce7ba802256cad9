// Paged GQA decode arithmetic on the vector ALU only (no matrix cores).  Kept as the measured
// alternative to the MFMA arithmetic; both run inside the same split-K kernel skeleton.
//
// A step's two 16-token blocks are processed one after the other.  Per block:
//   K granule [D/32][16][32]: lane l reads 16 bytes at (l + 64*i)*16, i.e. token l/4 and dims
//     32*i + 8*(l%4) .. +8.  Partial dot products (v_dot2_f32_bf16) of the G query heads are
//     summed over each lane quad (DPP), so all four lanes of a quad hold the token's scores.
//     The G query rows of the run live in a wave-private LDS tile (they are contiguous in q)
//     and are read back with 16-byte reads.
//   online softmax per head with a wave-wide max; probabilities go through a wave-private LDS
//     row so each lane can read the 4 it needs for its V piece.
//   V granule [4][D][4]: lane l reads 16 bytes at (l + 64*i)*16 = token quad (l + 64*i)/(D/2),
//     dims 2*m and 2*m+1 with m = (l + 64*i) % (D/2); fp32 FMAs into acc[g][0..1].  For D = 64
//     two lanes share a dim pair and are summed when a run ends.
#include "vox_decode_core.hpp"

namespace vox {
namespace {

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

__device__ inline float dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a),
                                         __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <int D, int G>
struct ValuMath {
  typedef int4 Desc;  // decode step descriptor, see the plan kernel
  __device__ static int ga(const Desc& d) { return d.x; }
  __device__ static int gb(const Desc& d) { return d.y; }
  __device__ static int meta(const Desc& d) { return d.z; }
  __device__ static int sigma(const Desc& d) { return d.w; }
  __device__ static int columns(const Params& p) { return p.G; }

  static constexpr int kBuffers = 2;
  static constexpr bool kDirect = false;  // every run leaves a partial record for the merge
  static constexpr int kStashFloats = 4096;  // 16 KB per wave: several decode records
  static constexpr int kMinWavesPerSimd = 2;
  static constexpr int NL = D / 32;  // 16-byte loads per lane per granule

  static constexpr int QCHUNKS = G * D / 8;                 // 16-byte pieces of the G query rows
  static constexpr int QPL = (QCHUNKS + kWave - 1) / kWave;  // pieces per lane

  struct Q {
    u32x4 r[QPL];
  };
  struct Regs {
    u32x4 k[2][NL], v[2][NL];
  };
  struct State {
    float m[G], l[G], acc[G][2];
  };

  const Params& p;
  int lane, tok, part;
  float (*p_lds)[kBlock];  // this wave's [G][16] probabilities
  u32x4* q_lds;            // this wave's [G][D/8] query slices

  __device__ ValuMath(int lane_, const Params& p_) : p(p_), lane(lane_) {
    __shared__ float lds_p[kWavesPerGroup][G][kBlock];
    __shared__ u32x4 lds_q[kWavesPerGroup][QCHUNKS];
    tok = lane >> 2;
    part = lane & 3;
    p_lds = lds_p[threadIdx.x >> 6];
    q_lds = lds_q[threadIdx.x >> 6];
  }

  // rows sigma*G .. sigma*G+G-1 of q are one contiguous run of QCHUNKS 16-byte pieces
  __device__ void load_q(Q& out, State&, const uint16_t* __restrict__ q, const Desc& dsc) const {
    const int sigma = dsc.w;
    const u32x4* src = reinterpret_cast<const u32x4*>(q + (size_t)sigma * G * D);
#pragma unroll
    for (int j = 0; j < QPL; ++j) {
      const int c = lane + kWave * j;
      out.r[j] = src[min(c, QCHUNKS - 1)];
    }
  }

  __device__ void install_q(State&, const Q& next) const {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < QPL; ++j) {
      const int c = lane + kWave * j;
      if (c < QCHUNKS) q_lds[c] = next.r[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }

  template <bool STREAM>
  __device__ void issue(Regs& r, const uint16_t* __restrict__ k_pool,
                        const uint16_t* __restrict__ v_pool, int ga, int gb) const {
    const size_t oa = (size_t)ga * (kBlock * D), ob = (size_t)gb * (kBlock * D);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      r.k[0][i] = kv_load<STREAM>(k_pool + oa + (lane + 64 * i) * 8);
      r.v[0][i] = kv_load<STREAM>(v_pool + oa + (lane + 64 * i) * 8);
    }
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      r.k[1][i] = kv_load<STREAM>(k_pool + ob + (lane + 64 * i) * 8);
      r.v[1][i] = kv_load<STREAM>(v_pool + ob + (lane + 64 * i) * 8);
    }
  }

  __device__ void reset(State& s) const {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      s.m[g] = -INFINITY;
      s.l[g] = 0.f;
      s.acc[g][0] = s.acc[g][1] = 0.f;
    }
  }

  __device__ void block(State& s, const u32x4 (&kb)[NL], const u32x4 (&vb)[NL], int ntok) const {
    const bool valid = tok < ntok;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const u32x4 qv = q_lds[g * (D / 8) + 4 * i + part];
        a = dot2(kb[i].x, qv.x, a);
        a = dot2(kb[i].y, qv.y, a);
        a = dot2(kb[i].z, qv.z, a);
        a = dot2(kb[i].w, qv.w, a);
      }
      a += dpp_f<0xB1>(a);  // lane quad: xor 1
      a += dpp_f<0x4E>(a);  //            xor 2
      const float sc = valid ? a * p.scale_log2 : -INFINITY;
      float mx = sc;  // max over the wave's 16 tokens
      mx = fmaxf(mx, dpp_f<0x141>(mx));
      mx = fmaxf(mx, dpp_f<0x140>(mx));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(s.m[g], mx);
      const float alpha = exp2f(s.m[g] - m_new);  // exp2(-inf) = 0 on the first block
      const float pr = exp2f(sc - m_new);
      s.l[g] = s.l[g] * alpha + pr;  // every lane of a quad carries its token's term
      s.m[g] = m_new;
      s.acc[g][0] *= alpha;
      s.acc[g][1] *= alpha;
      if (part == 0) p_lds[g][tok] = pr;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const bool tail = ntok < kBlock;  // wave-uniform
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int quad = (lane + kWave * i) / (D / 2);  // token quad of this 16-byte piece
      float v[8] = {bf16_lo(vb[i].x), bf16_hi(vb[i].x), bf16_lo(vb[i].y), bf16_hi(vb[i].y),
                    bf16_lo(vb[i].z), bf16_hi(vb[i].z), bf16_lo(vb[i].w), bf16_hi(vb[i].w)};
      if (tail) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (4 * quad + (e & 3) >= ntok) v[e] = 0.f;  // unread slots may hold NaN
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float4 pq = *reinterpret_cast<const float4*>(&p_lds[g][4 * quad]);
        float a0 = s.acc[g][0], a1 = s.acc[g][1];
        a0 = fmaf(pq.x, v[0], a0);
        a0 = fmaf(pq.y, v[1], a0);
        a0 = fmaf(pq.z, v[2], a0);
        a0 = fmaf(pq.w, v[3], a0);
        a1 = fmaf(pq.x, v[4], a1);
        a1 = fmaf(pq.y, v[5], a1);
        a1 = fmaf(pq.z, v[6], a1);
        a1 = fmaf(pq.w, v[7], a1);
        s.acc[g][0] = a0;
        s.acc[g][1] = a1;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  __device__ void compute(State& s, Regs& r, const Desc& dsc) const {
    const int ntok = dsc.z & kMetaTokMask;
    block(s, r.k[0], r.v[0], min(ntok, kBlock));
    if (ntok > kBlock) block(s, r.k[1], r.v[1], ntok - kBlock);
  }

  __device__ int used_columns(const Desc&) const { return G; }

  __device__ void finish(State& s, float* __restrict__ rec, float* __restrict__ ml) const {
    const int m = lane % (D / 2);  // dim pair owned by this lane
#pragma unroll
    for (int g = 0; g < G; ++g) {
      // every token's term sits in the four lanes of its quad: sum the wave and divide by 4
      float lsum = s.l[g];
      lsum += dpp_f<0xB1>(lsum);
      lsum += dpp_f<0x4E>(lsum);
      lsum += dpp_f<0x141>(lsum);
      lsum += dpp_f<0x140>(lsum);
      lsum += __shfl_xor(lsum, 16);
      lsum += __shfl_xor(lsum, 32);
      lsum *= 0.25f;
      if (lane == 0) *reinterpret_cast<float2*>(ml + 2 * g) = make_float2(s.m[g], lsum);
      float a0 = s.acc[g][0], a1 = s.acc[g][1];
      if (D == 64) {  // lanes l and l + 32 hold the same dim pair for different token quads
        a0 += __shfl_xor(a0, 32);
        a1 += __shfl_xor(a1, 32);
      }
      if (lane < D / 2) *reinterpret_cast<float2*>(rec + g * D + 2 * m) = make_float2(a0, a1);
    }
  }
};

template <int D>
hipError_t launch_g(const Params& p, int waves, const void* q, const void* k_pool,
                    const void* v_pool, const int32_t* header, const int4* desc, float2* pml,
                    float* pacc, hipStream_t st) {
  const unsigned grid = (unsigned)((waves + kWavesPerGroup - 1) / kWavesPerGroup);
#define VOX_VALU_CASE(GG)                                                                      \
  case GG:                                                                                     \
    hipLaunchKernelGGL((decode_kernel<ValuMath<D, GG>>), dim3(grid), dim3(256), 0, st, p,      \
                       (const uint16_t*)q, (const uint16_t*)k_pool, (const uint16_t*)v_pool,   \
                       header, desc, pml, pacc);                                               \
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

hipError_t launch_decode_valu(const Params& p, int waves, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* header, const int4* desc,
                              float2* partial_ml, float* partial_acc, hipStream_t st) {
  return p.D == 128 ? launch_g<128>(p, waves, q, k_pool, v_pool, header, desc, partial_ml,
                                    partial_acc, st)
                    : launch_g<64>(p, waves, q, k_pool, v_pool, header, desc, partial_ml,
                                   partial_acc, st);
}

}  // namespace vox
