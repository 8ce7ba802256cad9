// Paged GQA decode on the bf16 matrix cores (v_mfma_f32_16x16x32_bf16), one wave per
// (item, kv head), no LDS and no workgroup barriers: a wave streams its chunk of the context
// straight from the block pools into MFMA operand registers.
//
// Step = 32 tokens = logical blocks A, B of the chunk.  Lane l = (n = l % 16, c = l / 16).
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
//     carries p to ~2^-17 relative and the two partial outputs are added once at the end.
//   Output, D/16 tiles:   O_nt[16 dims x 16] += Vt_nt[16 dims x 32 tokens] * Pt[32 x 16]
//     A operand row i = dim 16*nt + i, k = 8*c + e: with the V granule [D][16] that is one
//     16-byte read (8 tokens of one dim) from block c>>1.  B operand = the lane's own 8
//     probabilities.  Nothing moves between lanes inside the loop except the max.
//     Result layout: lane (n, c), register r = dim 16*nt + 4*c + r of column n, so the
//     per-column rescale factor is lane-local.
#include "vox_common.hpp"

namespace vox {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// KV data is read exactly once per step: non-temporal loads keep it from displacing the
// block tables, queries and partial records in the caches.
__device__ inline u32x4 stream_load(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

__device__ inline uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
__device__ inline float round_bf16(float a) { return (float)(__bf16)a; }

template <int D, int NBUF>
__global__ __launch_bounds__(256, (NBUF <= 2 ? 2 : 1)) void decode_mfma_kernel(
    Params p, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ bt,
    const int32_t* __restrict__ lens, const int32_t* __restrict__ header,
    const Item* __restrict__ items, float2* __restrict__ pml, float* __restrict__ pacc) {
  constexpr int KK = D / 32;  // MFMAs per score tile
  constexpr int NT = D / 16;  // output dim tiles

  const int lane = threadIdx.x & (kWave - 1);
  const int wid = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6));
  if (wid >= header[0] * p.Hkv) return;
  const int item = wid / p.Hkv, h = wid % p.Hkv;
  const Item it = items[item];
  const int s = it.stream;
  const int nblk = it.nblocks;
  const int tok_first = it.first_block * kBlock;
  const int tok_end = min(lens[s], (it.first_block + nblk) * kBlock);
  const int nsteps = (nblk + 1) >> 1;
  const int n = lane & 15, c = lane >> 4;
  const int G = p.G;

  // Lane j keeps the physical id of chunk block j (clamped, so every id is a real block).
  const int my_id = bt[(size_t)s * p.max_nb + it.first_block + min(lane, nblk - 1)];

  // Query operand: column n -> head h*G + (n mod G) for n < 2G, zero otherwise.
  u32x4 qb[KK];
  {
    const bool has = n < 2 * G;
    const int head = h * G + (n < G ? n : n - G);
    const uint16_t* qrow = q + ((size_t)s * p.Hq + (has ? head : 0)) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qb[kk] = *reinterpret_cast<const u32x4*>(qrow + (c + 4 * kk) * 8);
      if (!has) qb[kk] = u32x4{0, 0, 0, 0};
    }
  }
  const bool is_lo = n >= G;

  // Per-lane element offsets inside a granule.
  const int k_tok = ((n >> 2) & 1) * 8 + (n & 3);  // + 4*T
  const int k_off = (c * kBlock + k_tok) * 8;       // + kk*4*16*8 + T*4*8
  const int v_off = n * kBlock + (c & 1) * 8;       // + nt*16*16
  const bool k_second = (n >> 3) != 0;              // K rows 8..15 come from block B
  const bool v_second = (c >> 1) != 0;              // lane groups 2,3 read block B

  u32x4 kr[NBUF][2 * KK], vr[NBUF][NT];
  f32x4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

#define VOX_ISSUE(ST, B)                                                                      \
  {                                                                                           \
    const int ja = 2 * (ST);                                                                  \
    const int id_a = __builtin_amdgcn_readlane(my_id, ja);                                    \
    const int id_b = __builtin_amdgcn_readlane(my_id, min(ja + 1, nblk - 1));                 \
    const uint16_t* kp = k_pool + granule_offset(k_second ? id_b : id_a, h, p.Hkv, D) + k_off; \
    const uint16_t* vp = v_pool + granule_offset(v_second ? id_b : id_a, h, p.Hkv, D) + v_off; \
    _Pragma("unroll") for (int kk = 0; kk < KK; ++kk) {                                       \
      kr[B][kk] = stream_load(kp + kk * (4 * kBlock * 8));                                    \
      kr[B][KK + kk] = stream_load(kp + kk * (4 * kBlock * 8) + 4 * 8);                       \
    }                                                                                         \
    _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                         \
        vr[B][nt] = stream_load(vp + nt * (16 * kBlock));                                     \
  }

#pragma unroll
  for (int b = 0; b < NBUF; ++b)
    if (b < nsteps) VOX_ISSUE(b, b)

  for (int st0 = 0; st0 < nsteps; st0 += NBUF) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
      const int st = st0 + b;
      if (st < nsteps) {
        // ---- scores
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          s0 = mfma(kr[b][kk], qb[kk], s0);
          s1 = mfma(kr[b][KK + kk], qb[kk], s1);
        }
        const int nvalid = tok_end - (tok_first + kStepTokens * st + 8 * c);  // may be <=0 or >=8
        float t[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          t[e] = e < nvalid ? t[e] * p.scale_log2 : -INFINITY;
          mx = fmaxf(mx, t[e]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite: lane group 0 always has a valid token
        const float alpha = exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        uint32_t pw[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float p0 = exp2f(t[e] - m_new), p1 = exp2f(t[e + 1] - m_new);
          psum += p0 + p1;
          const float h0 = round_bf16(p0), h1 = round_bf16(p1);
          pw[e >> 1] = is_lo ? pack_bf16(p0 - h0, p1 - h1) : pack_bf16(h0, h1);
        }
        l_run = l_run * alpha + psum;
        const u32x4 pb = {pw[0], pw[1], pw[2], pw[3]};
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) acc[nt] *= alpha;
        }
        // ---- unread slots of the tail may hold NaN/Inf bits: zero them (0 * NaN = NaN)
        if (tok_first + kStepTokens * (st + 1) > tok_end) {
          uint32_t msk[4];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            msk[j] = (2 * j < nvalid ? 0x0000FFFFu : 0u) | (2 * j + 1 < nvalid ? 0xFFFF0000u : 0u);
          const u32x4 mv = {msk[0], msk[1], msk[2], msk[3]};
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) vr[b][nt] &= mv;
        }
        // ---- output
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma(vr[b][nt], pb, acc[nt]);
        if (st + NBUF < nsteps) VOX_ISSUE(st + NBUF, b)
      }
    }
  }
#undef VOX_ISSUE

  // ---- partial record: sum over lane groups, hi + lo columns, then store
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  const bool writer = n < G;
  const size_t rec = (size_t)item * p.Hq + h * G + (writer ? n : 0);
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4 o;
#pragma unroll
    for (int r = 0; r < 4; ++r) o[r] = acc[nt][r] + __shfl(acc[nt][r], lane + G);
    if (writer) *reinterpret_cast<f32x4*>(pacc + rec * D + 16 * nt + 4 * c) = o;
  }
  if (writer && c == 0) pml[rec] = make_float2(m_run, l_run);
}

template <int D, int NBUF>
hipError_t launch_one(const Params& p, unsigned grid, const void* q, const void* k_pool,
                      const void* v_pool, const int32_t* bt, const int32_t* lens,
                      const int32_t* header, const Item* items, float2* pml, float* pacc,
                      hipStream_t st) {
  hipLaunchKernelGGL((decode_mfma_kernel<D, NBUF>), dim3(grid), dim3(256), 0, st, p,
                     (const uint16_t*)q, (const uint16_t*)k_pool, (const uint16_t*)v_pool, bt,
                     lens, header, items, pml, pacc);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_mfma(const Params& p, int max_wave_items, const void* q,
                              const void* k_pool, const void* v_pool, const int32_t* bt,
                              const int32_t* lens, const int32_t* header, const Item* items,
                              float2* partial_ml, float* partial_acc, hipStream_t st) {
  const unsigned grid = (unsigned)((max_wave_items + kWavesPerGroup - 1) / kWavesPerGroup);
  return p.D == 128 ? launch_one<128, 2>(p, grid, q, k_pool, v_pool, bt, lens, header, items,
                                         partial_ml, partial_acc, st)
                    : launch_one<64, 2>(p, grid, q, k_pool, v_pool, bt, lens, header, items,
                                        partial_ml, partial_acc, st);
}

}  // namespace vox
