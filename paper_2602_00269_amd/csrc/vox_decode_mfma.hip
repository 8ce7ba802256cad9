// Paged GQA decode arithmetic on the bf16 matrix cores: no LDS and no workgroup barriers, a
// wave streams KV granules from the block pools straight into MFMA operand registers.
//
// Step = 32 tokens = blocks A, B.  Lane l = (n = l % 16, c = l / 16).
//
//   Scores per block (v_mfma_f32_16x16x32_bf16, D/32 of them):
//       S[16 tokens x 16] = Kblk[16 x D] * Qt[D x 16]
//     A operand row n = token n, k-slice kk = dims 32*kk + 8*c .. +8: with the K granule
//     [D/32][16][32] that is the 16 bytes at kk*1024 + n*64 + c*16, so one load instruction
//     covers one contiguous KiB of one block.
//     B operand column n is a query head: columns [0,G) the G heads, [G,2G) the same heads
//     again, the rest zero.
//     Result: lane (n, c) holds, for its column, the scores of tokens 4*c + r of the block.
//   Softmax in log2 units per column over the step's 32 scores; the running max is shared by
//     the four lane groups.  Columns [0,G) keep hi = bf16(p); columns [G,2G) keep
//     lo = bf16(p - hi), so hi + lo carries p to ~2^-17 relative and the two partial outputs
//     are added once per run.
//   Output per step (the same 32-deep MFMA, D/16 of them, one per 16-dim tile):
//       O_tile[16 dims x 16] += Vt_tile[16 dims x 32 tokens] * Pt[32 tokens x 16]
//     The V granule [4][D][4] keeps four consecutive tokens of a dim adjacent: lane (n, c)
//     reads 16 bytes at c*D*8 + j*256 + n*16 = dims 32*j + 2*n and 32*j + 2*n + 1, tokens
//     4*c .. 4*c+3, of block A and of block B.  The low 8 bytes are row n of tile 2j, the
//     high 8 bytes row n of tile 2j+1 (tile 2j row i is dim 32j + 2i, tile 2j+1 row i is dim
//     32j + 2i + 1); reduction slots 0-3 of a lane group are its four tokens of block A,
//     slots 4-7 its four tokens of block B.  B operand = the lane's own 8 probabilities.
//     Nothing moves between lanes inside the loop except the max.
//     Result layout: lane (n, c), register r of tile 2j+u = dim 32j + 8c + 2r + u of column n,
//     so the per-column rescale factor is lane-local and a lane owns 8 consecutive dims.
#include "vox_decode_core.hpp"

namespace vox {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma32(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ inline uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
__device__ inline float round_bf16(float a) { return (float)(__bf16)a; }

// PACKED: the streams' query rows are packed rows q_rows[s] (mixed batches of the multi-token
// step) instead of rows s.
template <int D, int NBUF, bool PACKED = false>
struct MfmaMath {
  typedef int4 Desc;  // decode step descriptor, see the plan kernel
  __device__ static int ga(const Desc& d) { return d.x; }
  __device__ static int gb(const Desc& d) { return d.y; }
  __device__ static int meta(const Desc& d) { return d.z; }
  __device__ static int sigma(const Desc& d) { return d.w; }
  __device__ static int columns(const Params& p) { return p.G; }

  static constexpr int kBuffers = NBUF;
  static constexpr bool kDirect = false;  // every run leaves a partial record for the merge
  static constexpr int kStashFloats = 4096;  // 16 KB per wave: several decode records
  static constexpr int kMinWavesPerSimd = 1;
  static constexpr int KK = D / 32;  // score MFMAs per block = V loads per block
  static constexpr int NT = D / 16;  // output dim tiles

  struct Q {
    u32x4 b[KK];
  };
  struct Regs {
    u32x4 k[2][KK], v[2][KK];
  };
  struct State {
    Q q;
    f32x4 acc[NT];
    float m, l;
  };

  const Params& p;
  int lane, n, c, G;
  float lo_mul;  // 1 for the lo columns [G, 2G), 0 for the hi columns
  int k_off, v_off;

  __device__ MfmaMath(int lane_, const Params& p_) : p(p_), lane(lane_) {
    n = lane & 15;
    c = lane >> 4;
    G = p.G;
    lo_mul = n >= G ? 1.f : 0.f;
    k_off = n * 32 + c * 8;      // + kk * 512
    v_off = c * D * 4 + n * 8;   // + j * 128
  }

  // Query operand of segment sigma: column n -> row sigma*G + (n mod G) for n < 2G, else zero.
  __device__ void load_q(Q& out, State&, const uint16_t* __restrict__ q, const Desc& dsc) const {
    int sigma = dsc.w;
    if (PACKED) {  // (stream, kv head) -> (packed row, kv head)
      const int s = sigma / p.Hkv;
      sigma = p.q_rows[s] * p.Hkv + (sigma - s * p.Hkv);
    }
    const bool has = n < 2 * G;
    const int row = sigma * G + (has ? (n < G ? n : n - G) : 0);
    const uint16_t* qrow = q + (size_t)row * D + c * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      out.b[kk] = *reinterpret_cast<const u32x4*>(qrow + 32 * kk);
      if (!has) out.b[kk] = u32x4{0, 0, 0, 0};
    }
  }

  __device__ void install_q(State& s, const Q& next) const { s.q = next; }

  template <bool STREAM>
  __device__ void issue(Regs& r, const uint16_t* __restrict__ k_pool,
                        const uint16_t* __restrict__ v_pool, int ga, int gb) const {
    const uint16_t* ka = k_pool + (size_t)ga * (kBlock * D) + k_off;
    const uint16_t* kb = k_pool + (size_t)gb * (kBlock * D) + k_off;
    const uint16_t* va = v_pool + (size_t)ga * (kBlock * D) + v_off;
    const uint16_t* vb = v_pool + (size_t)gb * (kBlock * D) + v_off;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) r.k[0][kk] = kv_load<STREAM>(ka + kk * 512);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) r.k[1][kk] = kv_load<STREAM>(kb + kk * 512);
#pragma unroll
    for (int j = 0; j < KK; ++j) r.v[0][j] = kv_load<STREAM>(va + j * 128);
#pragma unroll
    for (int j = 0; j < KK; ++j) r.v[1][j] = kv_load<STREAM>(vb + j * 128);
  }

  __device__ void reset(State& s) const {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) s.acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    s.m = -INFINITY;
    s.l = 0.f;
  }

  __device__ void compute(State& s, Regs& r, const Desc& dsc) const {
    const int ntok = dsc.z & kMetaTokMask;
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      sa = mfma32(r.k[0][kk], s.q.b[kk], sa);
      sb = mfma32(r.k[1][kk], s.q.b[kk], sb);
    }
    float t[8] = {sa[0], sa[1], sa[2], sa[3], sb[0], sb[1], sb[2], sb[3]};
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] *= p.scale_log2;
    if (ntok < kStepTokens) {
      // Tail of a stream: slots past the last token may hold any bits (NaN/Inf included).
      // Their scores become -inf by selection, and their V values are cleared because
      // 0 * NaN = NaN.  A 16-byte V register is two dims x four tokens: dwords 0,2 hold tokens
      // 0,1 and dwords 1,3 hold tokens 2,3.
      const int va = ntok - 4 * c, vb = ntok - kBlock - 4 * c;  // valid among the lane's 4 + 4
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (e >= va) t[e] = -INFINITY;
        if (e >= vb) t[4 + e] = -INFINITY;
      }
      const auto mask4 = [](int valid) {
        const uint32_t lo = (0 < valid ? 0x0000FFFFu : 0u) | (1 < valid ? 0xFFFF0000u : 0u);
        const uint32_t hi = (2 < valid ? 0x0000FFFFu : 0u) | (3 < valid ? 0xFFFF0000u : 0u);
        return u32x4{lo, hi, lo, hi};
      };
      const u32x4 ma = mask4(va), mb = mask4(vb);
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        r.v[0][j] &= ma;
        r.v[1][j] &= mb;
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])),
                     fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(s.m, mx);  // finite: lane group 0 always holds a valid token
    // v_exp_f32 directly: arguments are <= 0 and results below 2^-126 may flush to zero
    const float alpha = __builtin_amdgcn_exp2f(s.m - m_new);
    s.m = m_new;
    float psum = 0.f;
    uint32_t pw[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const float p0 = __builtin_amdgcn_exp2f(t[e] - m_new);
      const float p1 = __builtin_amdgcn_exp2f(t[e + 1] - m_new);
      psum += p0 + p1;
      // hi columns keep bf16(p); lo columns keep bf16(p - bf16(p)): one fma with lo_mul = 0 / 1
      const float h0 = round_bf16(p0), h1 = round_bf16(p1);
      pw[e >> 1] = pack_bf16(fmaf(-lo_mul, h0, p0), fmaf(-lo_mul, h1, p1));
    }
    s.l = s.l * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) s.acc[nt] *= alpha;
    }
    // One 32-deep MFMA per 16-dim tile covers both blocks: reduction slots 0-3 of a lane group
    // are its four tokens of block A, slots 4-7 its four tokens of block B, for the V operand
    // and for the probabilities alike.
    const u32x4 pp = {pw[0], pw[1], pw[2], pw[3]};
#pragma unroll
    for (int j = 0; j < KK; ++j) {
      const u32x4 a = r.v[0][j], b = r.v[1][j];
      s.acc[2 * j] = mfma32(u32x4{a.x, a.y, b.x, b.y}, pp, s.acc[2 * j]);
      s.acc[2 * j + 1] = mfma32(u32x4{a.z, a.w, b.z, b.w}, pp, s.acc[2 * j + 1]);
    }
  }

  // Partial record of a run, written into the wave's LDS record.  The lo columns [G,2G) store
  // their accumulators first, the hi columns [0,G) then add their own on top (lane (n,c) and
  // lane (n+G,c) address the same floats), so no register shuffles are needed.  A lane owns
  // dims 32j + 8c .. +8 of its column: even ones in tile 2j, odd ones in tile 2j+1.
  __device__ int used_columns(const Desc&) const { return G; }

  __device__ void finish(State& s, float* __restrict__ rec, float* __restrict__ ml) const {
    float l = s.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const bool hi = n < G, lo = !hi && n < 2 * G;
    float* mine = rec + (hi ? n : n - G) * D + 8 * c;
    if (lo) {
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        const f32x4 e = s.acc[2 * j], o = s.acc[2 * j + 1];
        *reinterpret_cast<f32x4*>(mine + 32 * j) = f32x4{e[0], o[0], e[1], o[1]};
        *reinterpret_cast<f32x4*>(mine + 32 * j + 4) = f32x4{e[2], o[2], e[3], o[3]};
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (hi) {
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        const f32x4 e = s.acc[2 * j], o = s.acc[2 * j + 1];
        f32x4* d0 = reinterpret_cast<f32x4*>(mine + 32 * j);
        f32x4* d1 = reinterpret_cast<f32x4*>(mine + 32 * j + 4);
        *d0 = *d0 + f32x4{e[0], o[0], e[1], o[1]};
        *d1 = *d1 + f32x4{e[2], o[2], e[3], o[3]};
      }
      if (c == 0) *reinterpret_cast<float2*>(ml + 2 * n) = make_float2(s.m, l);
    }
  }
};

template <int D, int NBUF, bool PACKED = false>
hipError_t launch_one(const Params& p, int waves, const void* q, const void* k_pool,
                      const void* v_pool, const int32_t* header, const int4* desc, float2* pml,
                      float* pacc, hipStream_t st) {
  const unsigned grid = (unsigned)((waves + kWavesPerGroup - 1) / kWavesPerGroup);
  hipLaunchKernelGGL((decode_kernel<MfmaMath<D, NBUF, PACKED>>), dim3(grid), dim3(256), 0, st, p,
                     (const uint16_t*)q, (const uint16_t*)k_pool, (const uint16_t*)v_pool, header,
                     desc, pml, pacc);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_mfma(const Params& p, int waves, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* header, const int4* desc,
                              float2* partial_ml, float* partial_acc, hipStream_t st) {
  // Ring depth: three 32-token steps (48 KiB of loads in flight per wave) at head_dim 128, two
  // at head_dim 64 where deeper rings measured no faster.
  if (p.q_rows)
    return p.D == 128 ? launch_one<128, 3, true>(p, waves, q, k_pool, v_pool, header, desc,
                                                 partial_ml, partial_acc, st)
                      : launch_one<64, 2, true>(p, waves, q, k_pool, v_pool, header, desc,
                                                partial_ml, partial_acc, st);
  return p.D == 128 ? launch_one<128, 3>(p, waves, q, k_pool, v_pool, header, desc, partial_ml,
                                         partial_acc, st)
                    : launch_one<64, 2>(p, waves, q, k_pool, v_pool, header, desc, partial_ml,
                                        partial_acc, st);
}

}  // namespace vox
