// Paged GQA decode arithmetic on the bf16 matrix cores (v_mfma_f32_16x16x32_bf16): no LDS and
// no workgroup barriers, a wave streams KV granules from the block pools straight into MFMA
// operand registers.
//
// Step = 32 tokens = blocks A, B.  Lane l = (n = l % 16, c = l / 16).
//
//   Scores, two M-tiles T = 0, 1:   S_T[16 x 16] = Ktile_T[16 tokens x D] * Qt[D x 16]
//     A operand row i (= n when loading) is token 8*((i>>2)&1) + 4*T + (i&3) of block i>>3,
//     k-slice c + 4*kk of the dims.  With the K granule [D/8][16][8] each lane quad reads 64
//     contiguous bytes and the two tiles together cover both granules.
//     B operand column n is a query head: columns [0,G) the G heads, [G,2G) the same heads
//     again, the rest zero.
//     Result: lane (n, c) holds, for its column, the scores of tokens 8*c + e (e = 4*T + r)
//     of the step: eight consecutive tokens, all in block c>>1.
//   Softmax in log2 units per column; the running max is shared by the four lane groups.
//     Columns [0,G) keep hi = bf16(p); columns [G,2G) keep lo = bf16(p - hi), so hi + lo
//     carries p to ~2^-17 relative and the two partial outputs are added once per run.
//   Output, D/16 tiles:   O_nt[16 dims x 16] += Vt_nt[16 dims x 32 tokens] * Pt[32 x 16]
//     A operand row i = dim 16*nt + i, k = 8*c + e: with the V granule [D][16] that is one
//     16-byte read (8 tokens of one dim) from block c>>1.  B operand = the lane's own 8
//     probabilities.  Nothing moves between lanes inside the loop except the max.
//     Result layout: lane (n, c), register r = dim 16*nt + 4*c + r of column n, so the
//     per-column rescale factor is lane-local.
#include <stdlib.h>

#include "vox_decode_core.hpp"

namespace vox {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ inline uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
__device__ inline float round_bf16(float a) { return (float)(__bf16)a; }

template <int D, int NBUF>
struct MfmaMath {
  static constexpr int kBuffers = NBUF;
  static constexpr int kMinWavesPerSimd = NBUF <= 2 ? 2 : 1;
  static constexpr int KK = D / 32;  // MFMAs per score tile
  static constexpr int NT = D / 16;  // output dim tiles

  struct Q {
    u32x4 b[KK];
  };
  struct Regs {
    u32x4 k[2 * KK], v[NT];
  };
  struct State {
    Q q;
    f32x4 acc[NT];
    float m, l;
  };

  const Params& p;
  int lane, n, c, G;
  bool is_lo, k_second, v_second;
  int k_off, v_off;

  __device__ MfmaMath(int lane_, const Params& p_) : p(p_), lane(lane_) {
    n = lane & 15;
    c = lane >> 4;
    G = p.G;
    is_lo = n >= G;
    const int k_tok = ((n >> 2) & 1) * 8 + (n & 3);  // + 4*T
    k_off = (c * kBlock + k_tok) * 8;                 // + kk*4*16*8 + T*4*8
    v_off = n * kBlock + (c & 1) * 8;                 // + nt*16*16
    k_second = (n >> 3) != 0;                         // K rows 8..15 come from block B
    v_second = (c >> 1) != 0;                         // lane groups 2,3 read block B
  }

  // Query operand of segment sigma: column n -> row sigma*G + (n mod G) for n < 2G, else zero.
  __device__ void load_q(Q& out, const uint16_t* __restrict__ q, int sigma) const {
    const bool has = n < 2 * G;
    const int row = sigma * G + (has ? (n < G ? n : n - G) : 0);
    const uint16_t* qrow = q + (size_t)row * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      out.b[kk] = *reinterpret_cast<const u32x4*>(qrow + (c + 4 * kk) * 8);
      if (!has) out.b[kk] = u32x4{0, 0, 0, 0};
    }
  }

  __device__ void install_q(State& s, const Q& next) const { s.q = next; }

  template <bool STREAM>
  __device__ void issue(Regs& r, const uint16_t* __restrict__ k_pool,
                        const uint16_t* __restrict__ v_pool, int ga, int gb) const {
    const uint16_t* kp = k_pool + (size_t)(k_second ? gb : ga) * (kBlock * D) + k_off;
    const uint16_t* vp = v_pool + (size_t)(v_second ? gb : ga) * (kBlock * D) + v_off;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      r.k[kk] = kv_load<STREAM>(kp + kk * (4 * kBlock * 8));
      r.k[KK + kk] = kv_load<STREAM>(kp + kk * (4 * kBlock * 8) + 4 * 8);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) r.v[nt] = kv_load<STREAM>(vp + nt * (16 * kBlock));
  }

  __device__ void reset(State& s) const {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) s.acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    s.m = -INFINITY;
    s.l = 0.f;
  }

  __device__ void compute(State& s, Regs& r, int ntok) const {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      s0 = mfma(r.k[kk], s.q.b[kk], s0);
      s1 = mfma(r.k[KK + kk], s.q.b[kk], s1);
    }
    const int nvalid = ntok - 8 * c;  // valid tokens among this lane's eight; may be <=0 or >=8
    float t[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      t[e] = e < nvalid ? t[e] * p.scale_log2 : -INFINITY;
      mx = fmaxf(mx, t[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(s.m, mx);  // finite: lane group 0 always holds a valid token
    const float alpha = exp2f(s.m - m_new);
    s.m = m_new;
    float psum = 0.f;
    uint32_t pw[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const float p0 = exp2f(t[e] - m_new), p1 = exp2f(t[e + 1] - m_new);
      psum += p0 + p1;
      const float h0 = round_bf16(p0), h1 = round_bf16(p1);
      pw[e >> 1] = is_lo ? pack_bf16(p0 - h0, p1 - h1) : pack_bf16(h0, h1);
    }
    s.l = s.l * alpha + psum;
    const u32x4 pb = {pw[0], pw[1], pw[2], pw[3]};
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) s.acc[nt] *= alpha;
    }
    if (ntok < kStepTokens) {
      // Unread slots of a tail may hold NaN/Inf bits and 0 * NaN = NaN: clear them.
      uint32_t msk[4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        msk[j] = (2 * j < nvalid ? 0x0000FFFFu : 0u) | (2 * j + 1 < nvalid ? 0xFFFF0000u : 0u);
      const u32x4 mv = {msk[0], msk[1], msk[2], msk[3]};
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) r.v[nt] &= mv;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) s.acc[nt] = mfma(r.v[nt], pb, s.acc[nt]);
  }

  // Partial record of a run: sum over lane groups, add the hi and lo columns, store.
  __device__ void finish(State& s, int slot, float2* __restrict__ pml,
                         float* __restrict__ pacc) const {
    float l = s.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const bool writer = n < G;
    const size_t rec = (size_t)slot * G + (writer ? n : 0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      f32x4 o;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] = s.acc[nt][r] + __shfl(s.acc[nt][r], lane + G);
      if (writer) *reinterpret_cast<f32x4*>(pacc + rec * D + 16 * nt + 4 * c) = o;
    }
    if (writer && c == 0) pml[rec] = make_float2(s.m, l);
  }
};

template <int D, int NBUF>
hipError_t launch_one(const Params& p, int waves, const void* q, const void* k_pool,
                      const void* v_pool, const int32_t* header, const int4* desc, float2* pml,
                      float* pacc, hipStream_t st) {
  const unsigned grid = (unsigned)((waves + kWavesPerGroup - 1) / kWavesPerGroup);
  hipLaunchKernelGGL((decode_kernel<MfmaMath<D, NBUF>>), dim3(grid), dim3(256), 0, st, p,
                     (const uint16_t*)q, (const uint16_t*)k_pool, (const uint16_t*)v_pool, header,
                     desc, pml, pacc);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_mfma(const Params& p, int waves, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* header, const int4* desc,
                              float2* partial_ml, float* partial_acc, hipStream_t st) {
  static const int nbuf = getenv("VOX_NBUF") ? atoi(getenv("VOX_NBUF")) : 2;
#define VOX_GO(DD, NB) launch_one<DD, NB>(p, waves, q, k_pool, v_pool, header, desc, partial_ml, partial_acc, st)
  if (p.D == 128) return nbuf == 4 ? VOX_GO(128, 4) : nbuf == 3 ? VOX_GO(128, 3) : VOX_GO(128, 2);
  return nbuf == 4 ? VOX_GO(64, 4) : nbuf == 3 ? VOX_GO(64, 3) : VOX_GO(64, 2);
}

}  // namespace vox
