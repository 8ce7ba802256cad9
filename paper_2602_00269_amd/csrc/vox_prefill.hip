// Multi-token step: stream s brings n_s new tokens (a prompt, an admission chunk, a detokenizer
// chunk) that attend causally over its paged context.  The same split-K kernel skeleton as the
// decode step is used; what changes is the meaning of the 16 MFMA columns and the plan.
//
// A column group is TQ = 16 / G consecutive new tokens of one stream: their TQ x G (token, head)
// pairs fill the 16 columns of the score MFMAs, column n = j * G + g.  A tile is 1, 2, 4, 6 or 8
// column groups (chosen from the largest n_s) that share every loaded K/V step; segment (tile,
// kv head) walks the context [0, position of the tile's last token] in 32-token steps.  Column j may
// only see tokens up to its own position, which matters in the last steps of a segment only.
// Probabilities are split hi + lo as in the decode step, but as two output MFMAs per tile
// instead of duplicated columns.
#include <cfloat>

#include "vox_decode_core.hpp"

namespace vox {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kCols = 16;   // MFMA columns of one column group
constexpr int kBatch = 2;   // column groups whose stages are interleaved in one step

// Step descriptor of the multi-token step (32 bytes, wave-uniform).
//   a: granule of block A, granule of block B, meta (valid tokens | first | last), segment
//   b: first query row of the tile, tokens in the tile, cm0, kv head
//      cm0 = tokens of this step visible to column 0 (column j sees cm0 + j); >= 32: all
struct MqDesc {
  int4 a, b;
};

struct TileInfo {
  int32_t stream, q_row0, nq, pos0;
};

// A segment that was cut into several runs, for the merge: entry w of the list belongs to the
// segment whose first step lies in range w and that runs on past it (at most one per range);
// nruns == 0: no such segment.
struct SplitSegment {
  int32_t slot0, nruns;  // its partial records: slots slot0 .. slot0 + nruns - 1
  int32_t q_row0, nq;    // query rows of its tile
  int32_t h, pad0, pad1, pad2;
};

__device__ inline f32x4 mfma32(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// max(x of this lane, x of lane ^ 16) and the same for lane ^ 32, through the lane-swap
// instructions of gfx950 instead of a trip through LDS: after swapping the odd rows of 16
// lanes of one copy with the even rows of the other (or the upper 32 lanes with the lower 32),
// the two copies hold x of this lane's row and of its partner row, in one order or the other.
__device__ inline float max_across_16(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
constexpr float kMaxSlack = 8.f;

__device__ inline float max_across_32(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// QL: the query rows live in LDS (each lane's own copy, read back by the same lane, so no
// synchronisation is involved) instead of registers: room for more column groups per tile.
// REUSE: K/V loads are ordinary cacheable loads instead of streaming ones, for calls whose
// tiles walk the same context several times (prompts): later tiles then hit the caches.
template <int D, int NBUF, int NCG, bool QL = false, bool REUSE = false>
struct MqMath {
  typedef MqDesc Desc;
  __device__ static int ga(const Desc& d) { return d.a.x; }
  __device__ static int gb(const Desc& d) { return d.a.y; }
  __device__ static int meta(const Desc& d) { return d.a.z; }
  __device__ static int sigma(const Desc& d) { return d.a.w; }
  __device__ static int columns(const Params&) { return kCols * NCG; }

  static constexpr int kBuffers = NBUF;
  // a run that is its whole segment writes finished rows instead of a partial record
  static constexpr bool kDirect = true;
  // 39 KB per wave (all four waves: 156 of the CU's 160 KB): 4, 2, 1 records at head_dim 128
  // with 1, 2, 4 column groups; 9, 4, 2, 1 at head_dim 64 with 1, 2, 4, 8.  With the query rows
  // in LDS there is no room for records: they go straight to global memory.
  static constexpr int kStashFloats = QL ? 64 : 9984;
  static constexpr int kMinWavesPerSimd = 1;
  static constexpr int KK = D / 32;
  static constexpr int NT = D / 16;
  static constexpr int CB = QL ? 1 : (NCG < kBatch ? NCG : kBatch);  // groups per batch

  // The query rows of the next run are loaded straight into the state's registers right
  // after the last step of the previous run was computed (they are dead by then), ahead of
  // that step's refill and of the record stores, so the first step of the new run waits for
  // nothing younger than them.
  struct Q {};
  struct Regs {
    u32x4 k[2][KK], v[2][KK];
  };
  struct State {
    u32x4 q[QL ? 1 : NCG][KK];
    f32x4 acc[NCG][NT];
    float m[NCG], l[NCG];
  };

  const Params& p;
  int lane, n, c, jcol, gcol, tq;
  int k_off, v_off;
  u32x4* q_lds;  // QL: this lane's slot of entry (cg, kk) is q_lds[(cg * KK + kk) * 64]

  __device__ MqMath(int lane_, const Params& p_) : p(p_), lane(lane_) {
    if (QL) {
      __shared__ u32x4 q_mem[kWavesPerGroup][NCG * KK * kWave];
      q_lds = q_mem[threadIdx.x >> 6] + lane_;
    } else {
      q_lds = nullptr;
    }
    n = lane & 15;
    c = lane >> 4;
    tq = kCols / p.G;  // query tokens per column group
    jcol = n / p.G;    // token of this column inside its group (valid when < tq)
    gcol = n - jcol * p.G;
    k_off = n * 32 + c * 8;
    v_off = c * D * 4 + n * 8;
  }

  // Columns without a query row (tokens past the tile's last one, columns past tq * G) load
  // the tile's first row instead: every column is computed independently of the others and
  // the merge reads only the columns of real rows, so what they hold never matters.
  __device__ void load_group(u32x4 (&dst)[KK], const uint16_t* __restrict__ q, const Desc& d,
                             int cg) const {
    const int tok = cg * tq + jcol;
    const bool has = jcol < tq && tok < d.b.y;
    const int row = (d.b.x + (has ? tok : 0)) * p.Hq + d.b.w * p.G + (has ? gcol : 0);
    const uint16_t* qrow = q + (size_t)row * D + c * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) dst[kk] = *reinterpret_cast<const u32x4*>(qrow + 32 * kk);
  }

  __device__ void load_q(Q&, State& s, const uint16_t* __restrict__ q, const Desc& d) const {
    if (QL) {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) {
        u32x4 t[KK];
        load_group(t, q, d, cg);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) q_lds[(cg * KK + kk) * kWave] = t[kk];
      }
    } else {
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) load_group(s.q[cg], q, d, cg);
    }
  }

  __device__ u32x4 q_at(const State& s, int cg, int kk) const {
    return QL ? q_lds[(cg * KK + kk) * kWave] : s.q[QL ? 0 : cg][kk];
  }

  __device__ void install_q(State&, const Q&) const {}

  template <bool STREAM>
  __device__ void issue(Regs& r, const uint16_t* __restrict__ k_pool,
                        const uint16_t* __restrict__ v_pool, int ga_, int gb_) const {
    const uint16_t* ka = k_pool + (size_t)ga_ * (kBlock * D) + k_off;
    const uint16_t* kb = k_pool + (size_t)gb_ * (kBlock * D) + k_off;
    const uint16_t* va = v_pool + (size_t)ga_ * (kBlock * D) + v_off;
    const uint16_t* vb = v_pool + (size_t)gb_ * (kBlock * D) + v_off;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) r.k[0][kk] = kv_load<STREAM && !REUSE>(ka + kk * 512);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) r.k[1][kk] = kv_load<STREAM && !REUSE>(kb + kk * 512);
#pragma unroll
    for (int j = 0; j < KK; ++j) r.v[0][j] = kv_load<STREAM && !REUSE>(va + j * 128);
#pragma unroll
    for (int j = 0; j < KK; ++j) r.v[1][j] = kv_load<STREAM && !REUSE>(vb + j * 128);
  }

  __device__ void reset(State& s) const {
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) s.acc[cg][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      s.m[cg] = -INFINITY;
      s.l[cg] = 0.f;
    }
  }

  __device__ void compute(State& s, Regs& r, const Desc& d) const {
    const int ntok = d.a.z & kMetaTokMask;
    const int cm0 = d.b.z;
    // scores stay raw dot products until the exponent, exp2(raw * scale - max): the scale (times
    // log2 e, never zero) is applied by the same fused multiply-add that subtracts the maximum.
    // A hidden token gets the raw value whose product with the scale is -inf.
    const float scale = p.scale_log2;
    const bool positive = scale > 0.f;
    const float hidden = positive ? -INFINITY : INFINITY;
    if (ntok < kStepTokens) {
      // slots past the tile's last token may hold any bits: clear their V values (every
      // column's probability there is zero, and 0 * NaN = NaN)
      const int va = ntok - 4 * c, vb = ntok - kBlock - 4 * c;
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
    // Column groups are taken CB at a time, stage by stage, so that the latencies of one group
    // (dependent MFMAs, the two cross-lane maxima, the exponentials) hide behind the work of
    // the others: a single wave per SIMD has nobody else to switch to.
#pragma unroll
    for (int cg0 = 0; cg0 < NCG; cg0 += CB) {
      if (cg0 > 0 && cg0 * tq >= d.b.y) break;  // the tile's tokens end before this batch
      float t[CB][8];
#pragma unroll
      for (int b = 0; b < CB; ++b) {
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const u32x4 qv = q_at(s, cg0 + b, kk);
          sa = mfma32(r.k[0][kk], qv, sa);
          sb = mfma32(r.k[1][kk], qv, sb);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {  // raw dot products: the scale enters with the exponent
          t[b][e] = sa[e];
          t[b][4 + e] = sb[e];
        }
      }
      if (cm0 + cg0 * tq < kStepTokens) {
        // causal edge: the column of token j sees the first cm0 + j tokens of this step
#pragma unroll
        for (int b = 0; b < CB; ++b) {
          const int lim = cm0 + (cg0 + b) * tq + jcol;
          const int va = lim - 4 * c, vb = lim - kBlock - 4 * c;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (e >= va) t[b][e] = hidden;
            if (e >= vb) t[b][4 + e] = hidden;
          }
        }
      }
      // the largest scaled score of the lane is the scale times its largest or, under a
      // negative scale, smallest raw one
      float mx[CB];
      if (positive) {
#pragma unroll
        for (int b = 0; b < CB; ++b)
          mx[b] = fmaxf(fmaxf(fmaxf(t[b][0], t[b][1]), fmaxf(t[b][2], t[b][3])),
                        fmaxf(fmaxf(t[b][4], t[b][5]), fmaxf(t[b][6], t[b][7])));
      } else {
#pragma unroll
        for (int b = 0; b < CB; ++b)
          mx[b] = fminf(fminf(fminf(t[b][0], t[b][1]), fminf(t[b][2], t[b][3])),
                        fminf(fminf(t[b][4], t[b][5]), fminf(t[b][6], t[b][7])));
      }
#pragma unroll
      for (int b = 0; b < CB; ++b) mx[b] *= scale;
#pragma unroll
      for (int b = 0; b < CB; ++b) mx[b] = max_across_16(mx[b]);
#pragma unroll
      for (int b = 0; b < CB; ++b) mx[b] = max_across_32(mx[b]);
      float alpha[CB];
      uint32_t ph[CB][4], pl[CB][4];
      bool rescale = false;
#pragma unroll
      for (int b = 0; b < CB; ++b) {
        const int cg = cg0 + b;
        // The reference maximum of a column follows the scores lazily: it moves only when a
        // score exceeds it by more than kMaxSlack (in log2 units), so probabilities reach at
        // most 2^kMaxSlack and the accumulators are rescaled in the first steps of a run and
        // hardly ever after (a running maximum of random scores still grows, by little, in
        // most steps of a wave that carries 16 * CB columns).  The record's (max, sum,
        // accumulator) are all relative to this reference, which is all the merge asks for.
        const float m_new = mx[b] > s.m[cg] + kMaxSlack ? mx[b] : s.m[cg];
        // a column may have seen no token yet (its run starts past its causal limit): keep
        // the exponent arguments from being inf - inf, everything it contributes is zero
        const float m_ref = fmaxf(m_new, -FLT_MAX);
        alpha[b] = __builtin_amdgcn_exp2f(s.m[cg] - m_ref);
        rescale |= alpha[b] != 1.f;
        s.m[cg] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(t[b][e], scale, -m_ref));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(t[b][e + 1], scale, -m_ref));
          psum += p0 + p1;
          // hi = the upper 16 bits (truncation), lo = the exact remainder, truncated again:
          // hi + lo carries 16 significant bits of p
          const uint32_t b0 = __float_as_uint(p0), b1 = __float_as_uint(p1);
          const float l0 = p0 - __uint_as_float(b0 & 0xFFFF0000u);
          const float l1 = p1 - __uint_as_float(b1 & 0xFFFF0000u);
          ph[b][e >> 1] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
          pl[b][e >> 1] =
              __builtin_amdgcn_perm(__float_as_uint(l1), __float_as_uint(l0), 0x07060302u);
        }
        s.l[cg] = s.l[cg] * alpha[b] + psum;
      }
      if (__builtin_amdgcn_ballot_w64(rescale)) {
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) s.acc[cg0 + b][nt] *= alpha[b];
      }
      // one 32-deep MFMA per 16-dim tile covers both blocks (reduction slots 0-3: the lane
      // group's tokens of block A, 4-7: of block B), once for the hi and once for the lo part
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        const u32x4 va = r.v[0][j], vb = r.v[1][j];
        const u32x4 even = {va.x, va.y, vb.x, vb.y}, odd = {va.z, va.w, vb.z, vb.w};
#pragma unroll
        for (int b = 0; b < CB; ++b) {
          const u32x4 pph = {ph[b][0], ph[b][1], ph[b][2], ph[b][3]};
          s.acc[cg0 + b][2 * j] = mfma32(even, pph, s.acc[cg0 + b][2 * j]);
          s.acc[cg0 + b][2 * j + 1] = mfma32(odd, pph, s.acc[cg0 + b][2 * j + 1]);
        }
#pragma unroll
        for (int b = 0; b < CB; ++b) {
          const u32x4 ppl = {pl[b][0], pl[b][1], pl[b][2], pl[b][3]};
          s.acc[cg0 + b][2 * j] = mfma32(even, ppl, s.acc[cg0 + b][2 * j]);
          s.acc[cg0 + b][2 * j + 1] = mfma32(odd, ppl, s.acc[cg0 + b][2 * j + 1]);
        }
      }
    }
  }

  // Record: [16 * NCG columns][D] accumulators and as many (max, sum) pairs; column cg*16 + n.
  // A lane owns dims 32j + 8c .. +8 of its columns: even ones in tile 2j, odd ones in 2j+1.
  // whole column groups up to the tile's last token
  __device__ int used_columns(const Desc& d) const { return (d.b.y + tq - 1) / tq * kCols; }

  __device__ void finish(State& s, float* __restrict__ rec, float* __restrict__ ml) const {
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
      float l = s.l[cg];
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      float* mine = rec + (cg * kCols + n) * D + 8 * c;
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        const f32x4 e = s.acc[cg][2 * j], o = s.acc[cg][2 * j + 1];
        *reinterpret_cast<f32x4*>(mine + 32 * j) = f32x4{e[0], o[0], e[1], o[1]};
        *reinterpret_cast<f32x4*>(mine + 32 * j + 4) = f32x4{e[2], o[2], e[3], o[3]};
      }
      if (c == 0)
        *reinterpret_cast<float2*>(ml + 2 * (cg * kCols + n)) = make_float2(s.m[cg], l);
    }
  }

  // Rows of a run that was its whole segment, normalised: out = acc / sum and the log-sum-exp
  // (max + log2 sum) ln 2, what the merge of a single partial record would give.
  // Straight from the accumulators, as the step that ends the run: no trip through LDS.
  __device__ void finish_rows(State& s, const Desc& d) const {
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
      float l = s.l[cg];
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      const int tok = cg * tq + jcol;
      if (jcol >= tq || tok >= d.b.y) continue;
      const float inv = l > 0.f ? 1.f / l : 0.f;
      const size_t row = (size_t)(d.b.x + tok) * p.Hq + d.b.w * p.G + gcol;
      float* mine = p.out + row * D + 8 * c;
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        const f32x4 e = s.acc[cg][2 * j] * inv, o = s.acc[cg][2 * j + 1] * inv;
        *reinterpret_cast<f32x4*>(mine + 32 * j) = f32x4{e[0], o[0], e[1], o[1]};
        *reinterpret_cast<f32x4*>(mine + 32 * j + 4) = f32x4{e[2], o[2], e[3], o[3]};
      }
      if (p.lse && c == 0)
        p.lse[row] = l > 0.f ? (s.m[cg] + log2f(l)) * 0.69314718055994530942f : -INFINITY;
    }
  }
};

// ---------------------------------------------------------------------------------------
// Plan, two kernels.
//   plan:   per stream tiles_s = ceil(n_s / TQ) and steps_s = sum over its tiles of
//           ceil(ctx_tile / 32), exclusive scans PT (tiles) and PS (steps, per kv head); per
//           tile its first global step, step count and TileInfo; the waves' ranges.
//   expand: per tile the descriptors of its steps.
// New tokens of stream s as the plan sees them: in a mixed batch the streams that bring exactly
// one token are left to the decode kernels.
__device__ inline int planned_tokens(const Params& p, const int32_t* __restrict__ qo, int s) {
  const int n = qo[s + 1] - qo[s];
  return (p.skip_single && n == 1) ? 0 : n;
}
__device__ inline int tile_ctx(int L, int n, int tq, int tau) {
  return L - n + min(n, (tau + 1) * tq);  // tokens visible to the tile's last query
}
__device__ inline int steps_of(int ctx) { return (ctx + kStepTokens - 1) / kStepTokens; }

// Plan of the multi-token step, first part, one workgroup: (1) per-stream tile and step counts
// and their prefixes, (2) per tile its first step, step count and query rows, (3) the waves'
// ranges.  Each part needs the whole of the one before and is a chain of a few dependent
// look-ups per thread, so one workgroup that keeps the prefixes and the tile table in LDS
// (binary searches at LDS latency, no launch in between) is quicker than three launches.
constexpr int kPlanThreads = 1024;
constexpr int kPlanTilesLds = 6144;  // tile tables beyond this are searched in global memory

// Start of the run of segment sigma = t * Hkv + h on the global step axis.
__device__ inline int64_t segment_first(const int32_t* tile_first, const int32_t* tile_steps,
                                        int sigma, int Hkv) {
  const int t = sigma / Hkv, h = sigma - t * Hkv;
  return (int64_t)tile_first[t] + (int64_t)h * tile_steps[t];
}

// Ranges are balanced by cost rather than by step count.  A run costs its steps plus a fixed
// `run_cost` (in steps) for fetching its query rows and storing its record, which matters when
// runs are a few steps long (tiles of a short prompt): on the cost axis segment sigma occupies
// [first(sigma) + run_cost * sigma, ... + run_cost + steps(sigma)), overhead units first.
// Wave w starts at the step under cost w * quota, quota = ceil(total cost / waves); cost units
// inside an overhead zone map to the segment's first step, so a range can be empty but never
// lies strictly inside another segment's span of ranges.
__global__ __launch_bounds__(kPlanThreads) void mq_plan_kernel(
    Params p, int tq, const int32_t* __restrict__ lens, const int32_t* __restrict__ qo, int waves,
    int run_cost, int64_t desc_capacity, int32_t* __restrict__ header, int32_t* __restrict__ pt,
    int32_t* __restrict__ ps, int32_t* __restrict__ lens_single, int32_t* __restrict__ tile_first,
    int32_t* __restrict__ tile_steps, TileInfo* __restrict__ tile_info,
    int32_t* __restrict__ ranges, SplitSegment* __restrict__ split) {
  __shared__ int32_t s_pt[kMaxStreams + 1], s_ps[kMaxStreams + 1];
  __shared__ int32_t s_first[kPlanTilesLds + 1], s_steps[kPlanTilesLds];
  __shared__ int wave_tiles[kPlanThreads / kWave], wave_steps[kPlanThreads / kWave];
  __shared__ int s_N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int S = p.S;

  // (1) tiles and steps per stream, exclusive prefixes
  const int per = (S + kPlanThreads - 1) / kPlanThreads;
  const int lo = min(S, tid * per), hi = min(S, lo + per);
  int tiles = 0, steps = 0;
  for (int s = lo; s < hi; ++s) {
    const int L = lens[s], n = planned_tokens(p, qo, s);
    const int nt = (n + tq - 1) / tq;
    for (int tau = 0; tau < nt; ++tau) steps += steps_of(tile_ctx(L, n, tq, tau));
    tiles += nt;
  }
  int it = tiles, is = steps;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int a = __shfl_up(it, o), b = __shfl_up(is, o);
    if (lane >= o) {
      it += a;
      is += b;
    }
  }
  if (lane == kWave - 1) {
    wave_tiles[wv] = it;
    wave_steps[wv] = is;
  }
  __syncthreads();
  int bt_ = it - tiles, bs_ = is - steps;
  for (int k = 0; k < wv; ++k) {
    bt_ += wave_tiles[k];
    bs_ += wave_steps[k];
  }
  for (int s = lo; s < hi; ++s) {  // second walk writes the exclusive prefixes
    pt[s] = s_pt[s] = bt_;
    ps[s] = s_ps[s] = bs_;
    const int L = lens[s], n = planned_tokens(p, qo, s);
    const int nt = (n + tq - 1) / tq;
    for (int tau = 0; tau < nt; ++tau) bs_ += steps_of(tile_ctx(L, n, tq, tau));
    bt_ += nt;
    // mixed batch: the lengths as the decode kernels see them (streams with exactly one new
    // token keep theirs, all others become padded slots)
    if (lens_single) lens_single[s] = (qo[s + 1] - qo[s] == 1) ? L : 0;
  }
  if (tid == kPlanThreads - 1) {
    pt[S] = s_pt[S] = bt_;
    ps[S] = s_ps[S] = bs_;
    const int64_t n_all = (int64_t)bs_ * p.Hkv;
    const int64_t N = min(n_all, desc_capacity);
    header[kHdrSteps] = s_N = (int)N;
    header[kHdrPerWave] = (int)max((int64_t)1, (N + waves - 1) / waves);
    header[kHdrWaves] = waves;
    header[kHdrOverflow] = n_all > desc_capacity;
  }
  __syncthreads();

  // (2) the tile table
  const int total = s_pt[S];
  const bool in_lds = total <= kPlanTilesLds;
  for (int t = tid; t < total; t += kPlanThreads) {
    int a = 0, b = S;  // largest s with pt[s] <= t
    while (b - a > 1) {
      const int mid = (a + b) >> 1;
      if (s_pt[mid] <= t)
        a = mid;
      else
        b = mid;
    }
    const int s = a, tau = t - s_pt[s];
    const int L = lens[s], n = planned_tokens(p, qo, s);
    int cum = 0;
    for (int k = 0; k < tau; ++k) cum += steps_of(tile_ctx(L, n, tq, k));
    const int first = (s_ps[s] + cum) * p.Hkv, nsteps = steps_of(tile_ctx(L, n, tq, tau));
    tile_first[t] = first;
    tile_steps[t] = nsteps;
    if (in_lds) {
      s_first[t] = first;
      s_steps[t] = nsteps;
    }
    TileInfo info;
    info.stream = s;
    info.q_row0 = qo[s] + tau * tq;
    info.nq = min(tq, n - tau * tq);
    info.pos0 = L - n + tau * tq;
    tile_info[t] = info;
    if (t == total - 1) tile_first[total] = s_ps[S] * p.Hkv;
  }
  __syncthreads();  // the table is complete, in LDS or (same workgroup, same CU) in memory

  // (3) the waves' ranges
  const int32_t* first_of = in_lds ? s_first : tile_first;
  const int32_t* steps_of_tile = in_lds ? s_steps : tile_steps;
  const int launched = (waves + kWavesPerGroup - 1) / kWavesPerGroup * kWavesPerGroup;
  const int N = s_N;
  const int segments = total * p.Hkv;
  const int64_t all_cost = (int64_t)N + (int64_t)run_cost * segments;
  const int64_t quota = max((int64_t)1, (all_cost + waves - 1) / waves);
  for (int w = tid; w <= launched; w += kPlanThreads) {
    // waves past `waves` exist only to fill a workgroup: empty ranges
    if (w < waves) split[w].nruns = 0;  // the expand kernel fills in the cut segments
    const int64_t target = (int64_t)w * quota;
    if (w >= waves || target >= all_cost || segments == 0) {
      ranges[w] = N;
      continue;
    }
    int a = 0, b = segments;  // largest sigma whose cost interval starts at or before target
    while (b - a > 1) {
      const int mid = (a + b) >> 1;
      if (segment_first(first_of, steps_of_tile, mid, p.Hkv) + (int64_t)run_cost * mid <= target)
        a = mid;
      else
        b = mid;
    }
    const int64_t first = segment_first(first_of, steps_of_tile, a, p.Hkv);
    const int64_t into = target - (first + (int64_t)run_cost * a) - run_cost;
    const int64_t nsteps = steps_of_tile[a / p.Hkv];
    ranges[w] = (int)min((int64_t)N, first + min(nsteps, max((int64_t)0, into)));
  }
}

// The wave that owns step x is the largest w with ranges[w] <= x (empty ranges share their
// start with the next one, so the last of equal starts is the owner).
// Largest w in [lo, hi] with ranges[w] <= x, given ranges[lo] <= x.
__device__ inline int owner_between(const int32_t* ranges, int lo, int hi, int64_t x) {
  while (hi > lo) {
    const int mid = (lo + hi + 1) >> 1;
    if (ranges[mid] <= x)
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

// Workgroup (t, y) writes the descriptors of steps 256 y .. 256 y + 255 of tile t (all its kv
// heads, laid end to end): what a step needs of its tile is read once, and the owners of the
// tile's first and last step, found by each wave with 64 probes per round trip, bound every
// step's own search to the few ranges the tile spans.
__global__ __launch_bounds__(256) void mq_expand_kernel(
    Params p, const int32_t* __restrict__ bt, const int32_t* __restrict__ header,
    const int32_t* __restrict__ tile_first, const int32_t* __restrict__ tile_steps,
    const TileInfo* __restrict__ tile_info, const int32_t* __restrict__ ranges, int waves,
    MqDesc* __restrict__ desc, SplitSegment* __restrict__ split) {
  const int t = blockIdx.x, lane = threadIdx.x & (kWave - 1);
  const int N = header[kHdrSteps];
  const int f = tile_steps[t];
  const int64_t x0 = tile_first[t];
  const int total = (int)min((int64_t)f * p.Hkv, (int64_t)N - x0);  // steps with a descriptor
  if ((int)(blockIdx.y * blockDim.x) >= total) return;
  const TileInfo info = tile_info[t];
  // owners of the tile's first and last step: both searches advance together
  const int64_t x_last = x0 + total - 1;
  int a0 = 0, b0 = waves, a1 = 0, b1 = waves;
  while (b0 - a0 > 1 || b1 - a1 > 1) {
    const int s0 = (b0 - a0 + kWave - 1) / kWave, s1 = (b1 - a1 + kWave - 1) / kWave;
    const int i0 = a0 + lane * s0, i1 = a1 + lane * s1;
    const bool le0 = i0 < b0 && ranges[i0] <= x0, le1 = i1 < b1 && ranges[i1] <= x_last;
    const int h0 = __builtin_popcountll(__builtin_amdgcn_ballot_w64(le0));  // lane 0 always hits
    const int h1 = __builtin_popcountll(__builtin_amdgcn_ballot_w64(le1));
    a0 += (h0 - 1) * s0;
    b0 = min(b0, a0 + s0);
    a1 += (h1 - 1) * s1;
    b1 = min(b1, a1 + s1);
  }
  const int w_first = a0, w_last = a1;
  const int ctx = info.pos0 + info.nq;
  const int nb = (ctx + kBlock - 1) / kBlock;
  const int32_t* row = bt + (size_t)info.stream * p.max_nb;
  const int i = blockIdx.y * blockDim.x + threadIdx.x;
  if (i < total) {
    const int64_t x = x0 + i;
    const int h = i / f, st = i - h * f;
    const int ida = row[2 * st];
    const int idb = (2 * st + 1 < nb) ? row[2 * st + 1] : ida;
    int meta = min(kStepTokens, ctx - kStepTokens * st);
    const int w = owner_between(ranges, w_first, w_last, x);
    if (st == 0 || x == ranges[w]) meta |= kMetaFirst;
    if (st == f - 1 || x == ranges[w + 1] - 1) meta |= kMetaLast;
    // the segment's last step in the range that also holds its first: one run, no partial record
    if (st == f - 1 && x - st >= ranges[w]) meta |= kMetaWhole;
    MqDesc d;
    d.a = make_int4(ida * p.Hkv + h, idb * p.Hkv + h, meta, t * p.Hkv + h);
    d.b = make_int4(info.q_row0, info.nq, info.pos0 + 1 - kStepTokens * st, h);
    desc[x] = d;
    if (st == 0) {  // the segment's runs: waves w .. owner of its last step, slots w + sigma ..
      const int w1 = owner_between(ranges, w, w_last, min((int64_t)N, x + f) - 1);
      // a segment cut into several runs is the last one that starts in range w: entry w
      if (w1 > w) {
        SplitSegment e;
        e.slot0 = w + t * p.Hkv + h;
        e.nruns = w1 - w + 1;
        e.q_row0 = info.q_row0;
        e.nq = info.nq;
        e.h = h;
        e.pad0 = e.pad1 = e.pad2 = 0;
        split[w] = e;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Merge of the segments that were cut into several runs (the others wrote their rows
// themselves): workgroup (w, y) takes entry w of the list and column group y of its records;
// each of its four waves takes four of the group's 16 columns, one (query row, q head) per 16
// lanes, a lane D/16 consecutive dims.  Two passes over the runs' records: the largest maximum
// (16 runs at a time across the lanes), then the weighted sums (every lane of a column reads the
// run's (max, sum) itself; nothing moves between lanes there).
template <int D>
__global__ __launch_bounds__(256) void mq_merge_kernel(
    Params p, int ncg, const SplitSegment* __restrict__ split, const float2* __restrict__ pml,
    const float* __restrict__ pacc, float* __restrict__ out, float* __restrict__ lse) {
  constexpr int DPL = D / 16;  // dims per lane
  const SplitSegment e = split[blockIdx.x];
  if (e.nruns == 0) return;
  const int lane = threadIdx.x & (kWave - 1), l16 = lane & 15;
  const int col = blockIdx.y * kCols + (threadIdx.x >> 6) * 4 + (lane >> 4);
  const int tqg = kCols / p.G;  // tokens per column group
  const int nn = col & (kCols - 1), j = nn / p.G, g = nn - j * p.G;
  const int tok = blockIdx.y * tqg + j;
  const bool real = j < tqg && tok < e.nq;  // a column with a query row
  // columns without a row have no runs to walk (the 16 lanes of a column stay together, so
  // the shuffles below always find their partners)
  const int cols = kCols * ncg, n = real ? e.nruns : 0;
  const size_t rec0 = (size_t)e.slot0 * cols + col;
  float mx = -INFINITY, sum = 0.f;
  f32x4 acc[DPL / 4];
#pragma unroll
  for (int k = 0; k < DPL / 4; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int r0 = 0; r0 < n; r0 += 16) {
    const int r = r0 + l16;
    float m = r < n ? pml[rec0 + (size_t)r * cols].x : -INFINITY;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    mx = fmaxf(mx, m);
  }
#pragma unroll 4
  for (int r = 0; r < n; ++r) {
    const size_t rec = rec0 + (size_t)r * cols;
    const float2 ml = pml[rec];
    const f32x4* src = reinterpret_cast<const f32x4*>(pacc + rec * D + l16 * DPL);
    const float wgt = ml.x == -INFINITY ? 0.f : exp2f(ml.x - mx);
    sum += wgt * ml.y;
#pragma unroll
    for (int k = 0; k < DPL / 4; ++k) acc[k] += wgt * src[k];
  }
  if (!real) return;
  const float inv = sum > 0.f ? 1.f / sum : 0.f;
  const size_t w = (size_t)(e.q_row0 + tok) * p.Hq + e.h * p.G + g;
  f32x4* dst = reinterpret_cast<f32x4*>(out + w * D + l16 * DPL);
#pragma unroll
  for (int k = 0; k < DPL / 4; ++k) dst[k] = acc[k] * inv;
  if (lse && l16 == 0)
    lse[w] = sum > 0.f ? (mx + log2f(sum)) * 0.69314718055994530942f : -INFINITY;
}

// ---------------------------------------------------------------------------------------
// Multi-token append: one wave per new row, all kv heads of it (the search for the row's stream
// and the table entry are paid once per row, and every lane has bytes to move).
template <int D>
__global__ __launch_bounds__(256) void kv_append_multi_kernel(
    Params p, int total_q, const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
    uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool, const int32_t* __restrict__ bt,
    const int32_t* __restrict__ lens, const int32_t* __restrict__ qo) {
  const int lane = threadIdx.x & (kWave - 1);
  const int row = blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);
  if (row >= total_q) return;
  // largest s with qo[s] <= row, found by the whole wave: 64 probes per round trip to memory
  int a = 0, b = p.S;
  while (b - a > 1) {
    const int step = (b - a + kWave - 1) / kWave;
    const int idx = a + lane * step;
    const bool le = idx < b && qo[idx] <= row;
    const int hits = __builtin_popcountll(__builtin_amdgcn_ballot_w64(le));  // lane 0 always hits
    a += (hits - 1) * step;
    b = min(b, a + step);
  }
  const int s = a;
  const int n = qo[s + 1] - qo[s];
  const int pos = lens[s] - n + (row - qo[s]);
  if (pos < 0) return;
  const int64_t blk = bt[(int64_t)s * p.max_nb + (pos >> 4)];
  const int t = pos & (kBlock - 1);
  const uint16_t* krow = k_new + (size_t)row * p.Hkv * D;  // [Hkv][D] of this row
  const uint16_t* vrow = v_new + (size_t)row * p.Hkv * D;
  // K: 16 bytes per lane, D/8 lanes per head, 512/D heads per pass
  constexpr int kLanesK = D / 8, kHeadsK = kWave / kLanesK;
  for (int h0 = 0; h0 < p.Hkv; h0 += kHeadsK) {
    const int h = h0 + lane / kLanesK, d = (lane % kLanesK) * 8;
    if (h < p.Hkv)
      *reinterpret_cast<u32x4*>(k_pool + granule_offset(blk, h, p.Hkv, D) + k_elem(t, d)) =
          *reinterpret_cast<const u32x4*>(krow + h * D + d);
  }
  // V keeps four tokens of a dim together.  The row at the start of a quad whose other three
  // tokens are new as well writes the whole quad from the four rows; the other three rows of
  // such a quad skip V.  Quads that also hold older tokens, or end past the stream's last
  // token, are written one 2-byte element at a time (D/2 lanes per head, two dims each), so
  // bytes of tokens that are not being appended are never touched.
  const int j = row - qo[s];             // index among the stream's new tokens
  const int q0 = j - (t & 3);            // index of the quad's first token (may be < 0)
  const bool full_quad = q0 >= 0 && q0 + 3 < n;
  if (full_quad && (t & 3) != 0) return;
  const size_t stride = (size_t)p.Hkv * D;  // next new row of the same kv head
  if (full_quad) {
    // four rows x eight dims per lane in, the same 64 bytes transposed out (dim-major, the
    // quad's four tokens of a dim together): D/8 lanes per head, as for K
    for (int h0 = 0; h0 < p.Hkv; h0 += kHeadsK) {
      const int h = h0 + lane / kLanesK, d = (lane % kLanesK) * 8;
      if (h >= p.Hkv) continue;
      const uint16_t* src = vrow + h * D + d;
      u32x4 x[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) x[k] = *reinterpret_cast<const u32x4*>(src + k * stride);
      u32x4* dst = reinterpret_cast<u32x4*>(v_pool + granule_offset(blk, h, p.Hkv, D) +
                                            v_elem(t, d, D));
#pragma unroll
      for (int w = 0; w < 4; ++w) {  // word w of a row holds dims 2w and 2w + 1
        // low halves of tokens (0, 1) and (2, 3), then the high halves
        dst[w] = u32x4{__builtin_amdgcn_perm(x[1][w], x[0][w], 0x05040100u),
                       __builtin_amdgcn_perm(x[3][w], x[2][w], 0x05040100u),
                       __builtin_amdgcn_perm(x[1][w], x[0][w], 0x07060302u),
                       __builtin_amdgcn_perm(x[3][w], x[2][w], 0x07060302u)};
      }
    }
    return;
  }
  constexpr int kLanesV = D / 2, kHeadsV = kWave / kLanesV;
  for (int h0 = 0; h0 < p.Hkv; h0 += kHeadsV) {
    const int h = h0 + lane / kLanesV, d = (lane % kLanesV) * 2;
    if (h >= p.Hkv) continue;
    const uint32_t two = *reinterpret_cast<const uint32_t*>(vrow + h * D + d);
    uint16_t* dst = v_pool + granule_offset(blk, h, p.Hkv, D);
    dst[v_elem(t, d, D)] = (uint16_t)(two & 0xFFFFu);
    dst[v_elem(t, d + 1, D)] = (uint16_t)(two >> 16);
  }
}


}  // namespace

// Workspace map of the multi-token step (byte offsets), for `tiles` tiles at most, `slots`
// partial records, `desc_capacity` step descriptors and `waves` ranges.
PrefillWorkspace map_prefill_workspace(const Params& p, int ncg, int64_t tiles, int64_t slots,
                                       int64_t desc_capacity, int waves) {
  PrefillWorkspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  w.header = take(64 * sizeof(int32_t));
  // one entry per launched wave (whole workgroups) plus the end
  w.ranges = take(((size_t)waves + kWavesPerGroup + 1) * sizeof(int32_t));
  w.pt = take(((size_t)p.S + 1) * sizeof(int32_t));
  w.ps = take(((size_t)p.S + 1) * sizeof(int32_t));
  w.tile_first = take(((size_t)tiles + 1) * sizeof(int32_t));
  w.tile_steps = take((size_t)tiles * sizeof(int32_t));
  w.tile_info = take((size_t)tiles * sizeof(TileInfo));
  w.split_list = take(((size_t)waves + kWavesPerGroup + 1) * sizeof(SplitSegment));
  w.partial_ml = take((size_t)slots * kCols * ncg * sizeof(float2));
  w.partial_acc = take((size_t)slots * kCols * ncg * p.D * sizeof(float));
  w.desc = take((size_t)desc_capacity * sizeof(MqDesc));
  w.total = off;
  return w;
}

size_t prefill_desc_bytes() { return sizeof(MqDesc); }

hipError_t launch_kv_append_multi(const Params& p, int total_q, const void* k_new,
                                  const void* v_new, void* k_pool, void* v_pool,
                                  const int32_t* bt, const int32_t* lens, const int32_t* qo,
                                  hipStream_t st) {
  if (total_q <= 0) return hipSuccess;
  const unsigned grid = (unsigned)(((int64_t)total_q + kWavesPerGroup - 1) / kWavesPerGroup);
  if (p.D == 128)
    hipLaunchKernelGGL(kv_append_multi_kernel<128>, dim3(grid), dim3(256), 0, st, p, total_q,
                       (const uint16_t*)k_new, (const uint16_t*)v_new, (uint16_t*)k_pool,
                       (uint16_t*)v_pool, bt, lens, qo);
  else
    hipLaunchKernelGGL(kv_append_multi_kernel<64>, dim3(grid), dim3(256), 0, st, p, total_q,
                       (const uint16_t*)k_new, (const uint16_t*)v_new, (uint16_t*)k_pool,
                       (uint16_t*)v_pool, bt, lens, qo);
  return hipGetLastError();
}

int prefill_column_groups(const Params& p, int max_new_tokens) {
  const int tq = kCols / p.G;
  const int want = (max_new_tokens + tq - 1) / tq;  // groups the longest stream fills
  // Six groups (query rows in LDS, records straight to global memory) cost more per step than
  // four; they pay only where they save a second pass over the context: 5 or 6 groups wanted.
  if (p.D == 128 && want == 5) return 5;
  if (p.D == 128 && want == 6) return 6;
  // register budget: eight groups at head_dim 64, four at head_dim 128
  const int most = p.D == 64 ? 8 : 4;
  // fewest tiles first (each tile streams the context again), then the smallest kernel that
  // holds a tile: 15 tokens of 5 per group take one tile of four groups, not two of two
  const int tiles = (want + most - 1) / most;
  const int per_tile = tiles > 0 ? (want + tiles - 1) / tiles : 1;
  int ncg = 1;
  while (ncg < per_tile) ncg *= 2;
  return ncg;
}

template <int D, int NBUF, int NCG, bool QL = false, bool REUSE = false>
static void launch_mq(const Params& pk, unsigned grid, const void* q, const void* k_pool,
                      const void* v_pool, const int32_t* header, const MqDesc* desc, float2* pml,
                      float* pacc, hipStream_t st) {
  hipLaunchKernelGGL((decode_kernel<MqMath<D, NBUF, NCG, QL, REUSE>>), dim3(grid), dim3(256), 0, st, pk,
                     (const uint16_t*)q, (const uint16_t*)k_pool, (const uint16_t*)v_pool, header,
                     desc, pml, pacc);
}

hipError_t launch_prefill(const Params& p, const PrefillWorkspace& m, char* ws, int ncg,
                          int64_t tiles, int64_t steps, int64_t desc_capacity, int waves,
                          const void* q, const void* k_pool, const void* v_pool,
                          const int32_t* bt, const int32_t* lens, const int32_t* qo, float* out,
                          float* lse, hipStream_t st, hipEvent_t ev_before, hipEvent_t ev_after,
                          int phases, int64_t tile_streams, int32_t* lens_single,
                          int64_t max_tile_steps) {
  const int tq = (kCols / p.G) * ncg;  // query tokens per tile
  // most of the work re-reads contexts (several tiles per stream): keep K/V in the caches
  const bool reuse = tiles >= 4 * (tile_streams > 0 ? tile_streams : (int64_t)p.S);
  int32_t* header = (int32_t*)(ws + m.header);
  int32_t* pt = (int32_t*)(ws + m.pt);
  int32_t* ps = (int32_t*)(ws + m.ps);
  int32_t* tile_first = (int32_t*)(ws + m.tile_first);
  int32_t* tile_steps = (int32_t*)(ws + m.tile_steps);
  TileInfo* tile_info = (TileInfo*)(ws + m.tile_info);
  SplitSegment* split = (SplitSegment*)(ws + m.split_list);
  float2* pml = (float2*)(ws + m.partial_ml);
  float* pacc = (float*)(ws + m.partial_acc);
  MqDesc* desc = (MqDesc*)(ws + m.desc);
  int32_t* ranges = (int32_t*)(ws + m.ranges);
  // measured: a run boundary (query rows of the next run, record of the finished one) costs
  // about as much as four to six steps of a wave
  const int run_cost = 4;

  if (phases & kPrefillPlan)
    hipLaunchKernelGGL(mq_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, p, tq, lens, qo, waves,
                       run_cost, desc_capacity, header, pt, ps, lens_single, tile_first,
                       tile_steps, tile_info, ranges, split);
  if (tiles > 0 && (phases & kPrefillPlan)) {
    const dim3 eg((unsigned)tiles, (unsigned)((max_tile_steps + 255) / 256));
    hipLaunchKernelGGL(mq_expand_kernel, eg, dim3(256), 0, st, p, bt, header, tile_first,
                       tile_steps, tile_info, ranges, waves, desc, split);
  }
  if (tiles > 0 && (phases & kPrefillRun)) {
    const unsigned grid = (unsigned)((waves + kWavesPerGroup - 1) / kWavesPerGroup);
    Params pk = p;  // every wave reads its range from the table the plan wrote
    pk.n_steps = -1;
    pk.ranges_off = (int32_t)((m.ranges - m.header) / sizeof(int32_t));
    pk.out = out;
    pk.lse = lse;
    if (ev_before) (void)hipEventRecord(ev_before, st);
    if (p.D == 128) {
      if (ncg == 6)
        launch_mq<128, 2, 6, true>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else if (ncg == 5)
        launch_mq<128, 2, 5, true>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else if (ncg == 4 && reuse)
        launch_mq<128, 2, 4, false, true>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc,
                                          st);
      else if (ncg == 4)
        launch_mq<128, 2, 4>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else if (ncg == 2)
        launch_mq<128, 2, 2>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else
        launch_mq<128, 3, 1>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
    } else {
      if (ncg == 8 && reuse)
        launch_mq<64, 2, 8, false, true>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc,
                                         st);
      else if (ncg == 8)
        launch_mq<64, 2, 8>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else if (ncg == 4)
        launch_mq<64, 2, 4>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else if (ncg == 2)
        launch_mq<64, 2, 2>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
      else
        launch_mq<64, 2, 1>(pk, grid, q, k_pool, v_pool, header, desc, pml, pacc, st);
    }
    if (ev_after) (void)hipEventRecord(ev_after, st);
    // every range start cuts at most one segment: `waves` bounds the list
    const dim3 mg((unsigned)waves, (unsigned)ncg);
    if (p.D == 128)
      hipLaunchKernelGGL(mq_merge_kernel<128>, mg, dim3(256), 0, st, p, ncg, split, pml, pacc, out,
                         lse);
    else
      hipLaunchKernelGGL(mq_merge_kernel<64>, mg, dim3(256), 0, st, p, ncg, split, pml, pacc, out,
                         lse);
  }
  return hipGetLastError();
}

}  // namespace vox
