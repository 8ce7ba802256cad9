// Sampling step: logits -> next token per stream (repetition penalty, temperature, top-k, top-p,
// draw), one workgroup per stream (1024 threads, or 256 for vocabularies up to 16384 so that
// four streams share a CU), everything besides the logits in LDS.
//
// The token is decided by exact arithmetic: every float step is a single IEEE fp32 operation
// in a fixed order (contraction is off in this file's arithmetic helpers), softmax weights are
// 64-bit integers (2^40 * exp(-d) through a fixed polynomial), and all cumulative sums are
// integer sums, which do not depend on the order of addition.  Histograms can therefore be
// built with LDS atomics and the result is still reproducible bit for bit.
//
// Tokens are ranked by the composite key (bits of d = max - y, token id): 31 + 18 = 49 bits,
// unique per token.  Every cut the method needs is a position in that ranking where a running
// count or a running weight first reaches a threshold: the k-th token (top-k), the end of the
// shortest prefix holding top_p of the weight (top-p), the drawn token.  `locate` finds such a
// position by radix descent over the key: a histogram of (count, weight) per digit, a scan for
// the digit where the threshold is crossed, then the next digit inside that bucket.  The first
// digit's histogram is built once per stream and reused by every descent; once a bucket holds
// at most kCandidates tokens it is copied to LDS and the remaining digits never touch global
// memory again.  That is the general path.  Usually the cuts all lie among a few thousand
// tokens next to the maximum: the fast path in sample_kernel buckets tokens by distance,
// copies everything up to the first cut's bucket to LDS in one pass, sorts it there and reads
// the cuts off the running sums.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "vox.h"

namespace vox {
namespace {

constexpr int kIdBits = 18;  // vocabulary of at most 2^18 tokens
constexpr int kMaxVocab = 1 << kIdBits;
constexpr int kKeyBits = 31 + kIdBits;
constexpr int kLevels = 5;

// Workgroup shapes.  Results do not depend on them (the candidate limits only decide which of
// two equivalent paths runs); what differs is how much of a CU a stream takes.
struct AnyVocab {  // one workgroup per CU
  static constexpr int kThreads = 1024;
  static constexpr int kVocab = kMaxVocab;  // largest vocabulary: sizes the window bitmap
  static constexpr int kCandidates = 4096;  // tokens of a bucket / of the near range kept in LDS
  static constexpr int kBins = 2048;        // bins of a histogram: 2^(widest digit)
  // digits of the 49-bit key, most significant first: 11 + 10 + 10 + 9 + 9 bits
  static __device__ constexpr int width(int level) { return level == 0 ? 11 : level < 3 ? 10 : 9; }
  static __device__ constexpr int shift(int level) {
    return level == 0 ? 38 : level == 1 ? 28 : level == 2 ? 18 : level == 3 ? 9 : 0;
  }
};
struct SmallVocab {  // a few thousand tokens per stream are little work: a quarter of the
                     // threads and under 40 KB of LDS, so that four workgroups share a CU and a
                     // batch of a thousand streams is resident at once
  static constexpr int kThreads = 256;
  static constexpr int kVocab = 16384;
  static constexpr int kCandidates = 1536;
  static constexpr int kBins = 1024;
  // 10 + 10 + 10 + 10 + 9 bits
  static __device__ constexpr int width(int level) { return level < 4 ? 10 : 9; }
  static __device__ constexpr int shift(int level) { return level < 4 ? 39 - 10 * level : 0; }
};

// 2^40 * exp(-d): x = d * log2(e); n = floor(x), f = x - n; p = Taylor polynomial of 2^-f of
// degree 9 (Horner, fused multiply-adds); q = trunc(p * 2^24); result (q << 16) >> n.
__device__ inline uint64_t weight_of(float d) {
#pragma clang fp contract(off)
  // No branch: from x = 41 on the shift leaves nothing of q's 25 bits, so x is clamped to 63
  // (NaN included) and the result is zero as the definition asks for x >= 64.
  const float x0 = d * 0x1.715476p+0f;
  const float x = x0 < 63.0f ? x0 : 63.0f;
  const float nf = __builtin_floorf(x);
  const int n = (int)nf;
  const float f = x - nf;
  float p = -0x1.b5253ep-24f;
  p = __builtin_fmaf(p, f, 0x1.62c022p-20f);
  p = __builtin_fmaf(p, f, -0x1.ffcbfcp-17f);
  p = __builtin_fmaf(p, f, 0x1.430912p-13f);
  p = __builtin_fmaf(p, f, -0x1.5d87fep-10f);
  p = __builtin_fmaf(p, f, 0x1.3b2ab6p-7f);
  p = __builtin_fmaf(p, f, -0x1.c6b08ep-5f);
  p = __builtin_fmaf(p, f, 0x1.ebfbe0p-3f);
  p = __builtin_fmaf(p, f, -0x1.62e430p-1f);
  p = __builtin_fmaf(p, f, 1.0f);
  const uint64_t q = (uint64_t)(uint32_t)(p * 16777216.0f);
  return (q << 16) >> n;
}

struct StreamCtx {
  const float* z;        // this stream's logits
  const uint32_t* seen;  // LDS bitmap of the window's tokens, or nullptr
  int V;
  float r, invT, m;
};
// QUAD: the row is read four consecutive tokens per lane and load (its length is a multiple of
// four and its start 16-byte aligned: the host decides, one kernel per way of reading)
template <bool QUAD>
struct StreamCtxT : StreamCtx {
  static constexpr bool kQuad = QUAD;
};

// penalised, tempered logit of token v whose raw logit is z; `word` is word v / 32 of the
// window bitmap (zero when there is no window)
__device__ inline float tempered(const StreamCtx& c, int v, float z, uint32_t word) {
#pragma clang fp contract(off)
  float zp = z;
  if ((word >> (v & 31)) & 1u) zp = zp > 0.0f ? zp / c.r : zp * c.r;
  return zp * c.invT;
}

__device__ inline uint64_t key_of(const StreamCtx& c, int v, float z, uint32_t word,
                                  float* d_out) {
#pragma clang fp contract(off)
  const float d = c.m - tempered(c, v, z, word);
  *d_out = d;
  const uint64_t dkey = __builtin_bit_cast(uint32_t, d) & 0x7FFFFFFFu;
  return (dkey << kIdBits) | (uint32_t)v;
}

__device__ inline uint64_t key_from(float d, int v) {
  const uint64_t dkey = __builtin_bit_cast(uint32_t, d) & 0x7FFFFFFFu;
  return (dkey << kIdBits) | (uint32_t)v;
}
// d of a token outside the window: max - z / T
__device__ inline float plain_distance(const StreamCtx& c, float z) {
#pragma clang fp contract(off)
  const float y = z * c.invT;
  return c.m - y;
}

__device__ inline float d_of_key(uint64_t comp) {
  return __builtin_bit_cast(float, (uint32_t)(comp >> kIdBits));
}

struct Located {
  uint64_t comp;                   // key of the token at the crossing
  uint64_t through_cnt, through_mass;  // tokens / weight up to and including it
};

constexpr float kBucketsPerUnit = 64.0f;
constexpr float kNearRange = 8.0f;
constexpr int kNearBuckets = 512;  // kNearRange * kBucketsPerUnit


__device__ inline int bucket_of(float d) { return (int)(d * kBucketsPerUnit); }  // d in [0, kCountRange)

// First index i in [0, n) with cum[i] >= thr (n if none).
__device__ inline int first_reaching(const unsigned long long* cum, int n,
                                     unsigned long long thr) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (cum[mid] >= thr)
      hi = mid;
    else
      lo = mid + 1;
  }
  return lo;
}

// Everything that depends on the workgroup shape, as static members of a class template (laid
// out like a namespace: members are not indented).
template <class Cfg>
struct Sampler {
static constexpr int kThreads = Cfg::kThreads;
static constexpr int kWaves = kThreads / 64;
static constexpr int kCandidates = Cfg::kCandidates;
static constexpr int kSuperset = Cfg::kCandidates;
static constexpr int kBins = Cfg::kBins;
static constexpr float kCountRange = kBins / kBucketsPerUnit;  // counts are kept out to here

// Calls f(v, z[v], bitmap word of v) for every token of the stream, this thread's share, in
// no particular order (nothing the callers compute depends on it); the logits of several
// tokens are loaded before any of them is used, so the loads overlap (more of them for light
// bodies, fewer where the body needs the registers).  Rows read in quads: twice the tokens in
// flight with half the loads, and the four tokens share one look-up of the bitmap.
template <int kAhead = 4, class Ctx, class F>
static __device__ inline void for_each_token(const Ctx& c, F f) {
  if constexpr (Ctx::kQuad) {
    const float4* z4 = reinterpret_cast<const float4*>(c.z);
    const int quads = c.V >> 2;
    constexpr int kQuadsAhead = kAhead >= 2 ? kAhead / 2 : 1;
    for (int q0 = threadIdx.x; q0 < quads; q0 += kThreads * kQuadsAhead) {
      float4 z[kQuadsAhead];
#pragma unroll
      for (int e = 0; e < kQuadsAhead; ++e) {
        const int q = q0 + e * kThreads;
        z[e] = q < quads ? z4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int e = 0; e < kQuadsAhead; ++e) {
        const int q = q0 + e * kThreads;
        if (q < quads) {
          const int v = 4 * q;
          const uint32_t word = c.seen ? c.seen[v >> 5] : 0u;
          f(v, z[e].x, word);
          f(v + 1, z[e].y, word);
          f(v + 2, z[e].z, word);
          f(v + 3, z[e].w, word);
        }
      }
    }
  } else {
    for (int v0 = threadIdx.x; v0 < c.V; v0 += kThreads * kAhead) {
      float z[kAhead];
#pragma unroll
      for (int e = 0; e < kAhead; ++e) {
        const int v = v0 + e * kThreads;
        z[e] = v < c.V ? c.z[v] : 0.0f;
      }
#pragma unroll
      for (int e = 0; e < kAhead; ++e) {
        const int v = v0 + e * kThreads;
        if (v < c.V) f(v, z[e], c.seen ? c.seen[v >> 5] : 0u);
      }
    }
  }
}

// Calls f(v, four logits from token v on, bitmap word of v) for this thread's quads of a row
// read in quads; the next quads are requested before the current ones are worked on.
template <class Ctx, class F>
static __device__ inline void for_each_quad(const Ctx& c, F f) {
  constexpr int kQuads = 1;  // measured: more quads per turn do not pay, the pass is bound by its arithmetic
  const float4* z4 = reinterpret_cast<const float4*>(c.z);
  const int quads = c.V >> 2;
  if (quads <= 0) return;
  // a quad past the end is never used: its load reads the row's last quad instead, so that
  // every load is one unconditional 16-byte access
  const int last = quads - 1;
  float4 cur[kQuads], next[kQuads];
#pragma unroll
  for (int e = 0; e < kQuads; ++e) cur[e] = z4[min((int)threadIdx.x + e * kThreads, last)];
  for (int q0 = threadIdx.x; q0 < quads; q0 += kThreads * kQuads) {
#pragma unroll
    for (int e = 0; e < kQuads; ++e) next[e] = z4[min(q0 + (kQuads + e) * kThreads, last)];
#pragma unroll
    for (int e = 0; e < kQuads; ++e) {
      const int q = q0 + e * kThreads;
      if (q < quads) f(4 * q, cur[e], c.seen ? c.seen[q >> 3] : 0u);
    }
#pragma unroll
    for (int e = 0; e < kQuads; ++e) cur[e] = next[e];
  }
}

struct Lds {
  uint32_t seen[Cfg::kVocab / 32];
  uint32_t cnt[kBins], cnt0[kBins];
  unsigned long long mass[2 * kBins];  // [0, kBins): histogram in use; [kBins, 2 kBins): level 0
  unsigned long long cand[kCandidates];
  unsigned long long wave_cnt[kWaves], wave_mass[kWaves];
  float wave_max[kWaves];
  // result of a scan
  int bin;
  unsigned long long before_cnt, before_mass, total_cnt, total_mass;
  uint32_t n_cand;
};

// Finds, over bins [0, nbins), the first bin where the running count (by_mass = false) or
// running weight reaches thr; leaves the bin and the sums before it in LDS.  All threads call.
static __device__ inline void scan_bins(Lds& s, const uint32_t* cnt, const unsigned long long* mass,
                                 int nbins, bool by_mass, unsigned long long thr) {
  constexpr int kPerThread = kBins / kThreads;  // consecutive bins per thread
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int b0 = kPerThread * tid;
  unsigned long long c[kPerThread], m[kPerThread], tc = 0, tm = 0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    c[e] = b0 + e < nbins ? cnt[b0 + e] : 0;
    m[e] = b0 + e < nbins ? mass[b0 + e] : 0;
    tc += c[e];
    tm += m[e];
  }
  unsigned long long ic = tc, im = tm;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long ac = __shfl_up(ic, o), am = __shfl_up(im, o);
    if (lane >= o) {
      ic += ac;
      im += am;
    }
  }
  if (lane == 63) {
    s.wave_cnt[wv] = ic;
    s.wave_mass[wv] = im;
  }
  if (tid == 0) s.bin = -1;
  __syncthreads();
  unsigned long long ec = ic - tc, em = im - tm;  // exclusive, inside the wave
  for (int k = 0; k < wv; ++k) {
    ec += s.wave_cnt[k];
    em += s.wave_mass[k];
  }
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {  // running value before and after bin b0 + e
    const unsigned long long before = by_mass ? em : ec;
    const unsigned long long after = before + (by_mass ? m[e] : c[e]);
    if (before < thr && thr <= after) {
      s.bin = b0 + e;
      s.before_cnt = ec;
      s.before_mass = em;
    }
    ec += c[e];
    em += m[e];
  }
  if (tid == kThreads - 1) {
    s.total_cnt = ec;
    s.total_mass = em;
  }
  __syncthreads();
}

static __device__ inline void clear_hist(Lds& s) {
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    s.cnt[b] = 0;
    s.mass[b] = 0;
  }
  __syncthreads();
}

// Position where the running count / weight first reaches thr (1 <= thr <= total).
template <class Ctx>
static __device__ Located locate(Lds& s, const Ctx& c, bool by_mass, unsigned long long thr) {
  uint64_t prefix = 0;  // the digits chosen so far, right-aligned
  int prefix_bits = 0;
  unsigned long long before_cnt = 0, before_mass = 0, bucket_mass = 0;
  bool in_lds = false;
  uint32_t n_cand = 0;
  for (int level = 0; level < kLevels; ++level) {
    const int width = Cfg::width(level), shift = Cfg::shift(level);
    const uint32_t* cnt = s.cnt;
    const unsigned long long* mass = s.mass;
    if (level == 0) {  // built once per stream
      cnt = s.cnt0;
      mass = s.mass + kBins;
    } else {
      clear_hist(s);
      const uint32_t digit_mask = (1u << width) - 1;
      if (in_lds) {
        for (uint32_t i = threadIdx.x; i < n_cand; i += kThreads) {
          const uint64_t comp = s.cand[i];
          if ((comp >> (kKeyBits - prefix_bits)) != prefix) continue;
          const uint32_t b = (uint32_t)(comp >> shift) & digit_mask;
          atomicAdd(&s.cnt[b], 1u);
          atomicAdd(&s.mass[b], (unsigned long long)weight_of(d_of_key(comp)));
        }
      } else {
        for_each_token(c, [&](int v, float z, uint32_t word) {
          float d;
          const uint64_t comp = key_of(c, v, z, word, &d);
          if ((comp >> (kKeyBits - prefix_bits)) != prefix) return;
          const uint32_t b = (uint32_t)(comp >> shift) & digit_mask;
          atomicAdd(&s.cnt[b], 1u);
          atomicAdd(&s.mass[b], (unsigned long long)weight_of(d));
        });
      }
      __syncthreads();
    }
    scan_bins(s, cnt, mass, 1 << width, by_mass, thr - (by_mass ? before_mass : before_cnt));
    const int b = s.bin;  // >= 0: thr is within the total of the bucket being refined
    before_cnt += s.before_cnt;
    before_mass += s.before_mass;
    const uint32_t bucket_cnt = cnt[b];
    bucket_mass = mass[b];
    prefix = (prefix << width) | (uint32_t)b;
    prefix_bits += width;
    __syncthreads();  // every thread has read the scan result
    if (!in_lds && level + 1 < kLevels && bucket_cnt <= (uint32_t)kCandidates) {
      // copy the bucket's keys to LDS; later digits are read from there
      if (threadIdx.x == 0) s.n_cand = 0;
      __syncthreads();
      for_each_token(c, [&](int v, float z, uint32_t word) {
        float d;
        const uint64_t comp = key_of(c, v, z, word, &d);
        if ((comp >> (kKeyBits - prefix_bits)) == prefix) s.cand[atomicAdd(&s.n_cand, 1u)] = comp;
      });
      __syncthreads();
      n_cand = s.n_cand;
      in_lds = true;
    }
  }
  // all 49 bits chosen: the bucket is one token
  Located out;
  out.comp = prefix;
  out.through_cnt = before_cnt + 1;
  out.through_mass = before_mass + bucket_mass;
  return out;
}

// Per-stream set-up: the window's tokens as an LDS bitmap, 1/T, the maximum tempered logit.
template <class Ctx>
static __device__ Ctx open_stream(Lds& s, int V, const float* __restrict__ logits,
                                 const vox_sampling_t& prm, const int32_t* __restrict__ history,
                                 int window, int stream) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  Ctx c;
  c.z = logits + (size_t)stream * V;
  c.V = V;
  c.r = prm.repetition_penalty;
  c.invT = (prm.temperature > 0.0f) ? 1.0f / prm.temperature : 1.0f;
  c.seen = nullptr;
  if (window > 0) {
    // the first window entries are requested before the barrier, not after it
    const int32_t first = tid < window ? history[(size_t)stream * window + tid] : -1;
    for (int i = tid; i < (V + 31) / 32; i += kThreads) s.seen[i] = 0;
    __syncthreads();
    if (first >= 0 && first < V) atomicOr(&s.seen[first >> 5], 1u << (first & 31));
    for (int j = tid + kThreads; j < window; j += kThreads) {
      const int32_t v = history[(size_t)stream * window + j];
      if (v >= 0 && v < V) atomicOr(&s.seen[v >> 5], 1u << (v & 31));
    }
    __syncthreads();
    c.seen = s.seen;
  }
  c.m = 0.0f;
  float mx = -INFINITY;
  for_each_token<Ctx::kQuad ? 8 : 16>(
      c, [&](int v, float z, uint32_t word) { mx = fmaxf(mx, tempered(c, v, z, word)); });
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if (lane == 0) s.wave_max[wv] = mx;
  __syncthreads();
  mx = s.wave_max[0];
  for (int k = 1; k < kWaves; ++k) mx = fmaxf(mx, s.wave_max[k]);
  c.m = mx;
  return c;
}

// Verification aid: the distance d = max - y and the integer weight of every token.
static __device__ void weights_body(int V, const float* __restrict__ logits,
                                    const vox_sampling_t* __restrict__ params,
                                    const int32_t* __restrict__ history, int window,
                                    float* __restrict__ d_out,
                                    unsigned long long* __restrict__ w_out) {
  __shared__ Lds s;
  const int stream = blockIdx.x;
  const auto c =
      open_stream<StreamCtxT<false>>(s, V, logits, params[stream], history, window, stream);
  for_each_token(c, [&](int v, float z, uint32_t word) {
    float d;
    (void)key_of(c, v, z, word, &d);
    d_out[(size_t)stream * V + v] = d;
    w_out[(size_t)stream * V + v] = weight_of(d);
  });
}

// Level-0 histogram of the radix descent (digits of the key), for the general path.
template <class Ctx>
static __device__ void build_key_histogram(Lds& s, const Ctx& c) {
  for (int b = threadIdx.x; b < kBins; b += kThreads) {
    s.cnt0[b] = 0;
    s.mass[kBins + b] = 0;
  }
  __syncthreads();
  for_each_token(c, [&](int v, float z, uint32_t word) {
    float d;
    const uint64_t comp = key_of(c, v, z, word, &d);
    const uint32_t b = (uint32_t)(comp >> Cfg::shift(0));
    atomicAdd(&s.cnt0[b], 1u);
    const unsigned long long w = weight_of(d);
    if (w) atomicAdd(&s.mass[kBins + b], w);
  });
  __syncthreads();
}

// General path: every cut by radix descent over the whole vocabulary.  It may be compiled as a
// real call, so everything goes in and comes out by value: an argument passed by address would
// make the caller keep that object in memory, and store it, on the fast path too.
struct Picked {
  int token, n_kept;
};
template <class Ctx>
static __device__ Picked sample_general(Lds& s, const Ctx c, const float top_p, const int top_k,
                                        bool greedy, float u) {
  build_key_histogram(s, c);
  if (greedy) return {(int)(locate(s, c, false, 1).comp & (kMaxVocab - 1)), 1};
  unsigned long long total;
  unsigned long long n = (unsigned long long)c.V;
  if (top_k > 0 && top_k < c.V) {
    const Located k = locate(s, c, false, (unsigned long long)top_k);
    n = (unsigned long long)top_k;
    total = k.through_mass;
  } else {
    scan_bins(s, s.cnt0, s.mass + kBins, kBins, false, ~0ull);  // no crossing: totals only
    total = s.total_mass;
    __syncthreads();
  }
  if (top_p < 1.0f) {
    unsigned long long thr = (unsigned long long)((double)top_p * (double)total);
    if (thr < 1) thr = 1;
    const Located pcut = locate(s, c, true, thr);
    n = pcut.through_cnt;
    total = pcut.through_mass;
  }
  const unsigned long long target = (unsigned long long)((double)u * (double)total);
  return {(int)(locate(s, c, true, target + 1).comp & (kMaxVocab - 1)), (int)n};
}

// Fast path.  The cuts almost always lie among the few tokens next to the maximum.  In the same
// pass that adds up every token's weight, the tokens with d < kNearRange are bucketed by
// distance (64 buckets per unit of d) and copied to LDS.  If there are at most kSuperset of
// them and the first cut that is needed (top-k by count, else top-p, else the draw itself, by
// weight) falls inside their buckets, every later cut does too (each lies at or before the
// previous one): the copies are sorted by key and the cuts are searches in the running sums of
// their weights.  Otherwise the general path starts over.
template <bool QUAD>
static __device__ void sample_body(
    int V, const float* __restrict__ logits, const vox_sampling_t* __restrict__ params,
    const int32_t* __restrict__ history, int window, const float* __restrict__ uniforms,
    int32_t* __restrict__ tokens, int32_t* __restrict__ kept) {
  __shared__ Lds s;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int stream = blockIdx.x;
  const vox_sampling_t prm = params[stream];
  const bool greedy = !(prm.temperature > 0.0f);
  const float u = uniforms[stream];
  const auto c = open_stream<StreamCtxT<QUAD>>(s, V, logits, prm, history, window, stream);
  // One pass over the logits: tokens within kNearRange of the maximum go into the bucket
  // histogram and into the candidate list, all others only add to the thread's weight total
  // (and, when a top-k cut is wanted, to the bucket counts out to kCountRange, since the k-th
  // token of a peaked distribution can lie farther out than the near range).
  const bool use_k = !greedy && prm.top_k > 0 && prm.top_k < V;
  const bool use_p = !greedy && prm.top_p < 1.0f;
  const int count_buckets = use_k ? kBins : kNearBuckets;
  for (int b = tid; b < count_buckets; b += kThreads) {
    s.cnt0[b] = 0;
    s.mass[kBins + b] = 0;  // only the near buckets receive weight
  }
  if (tid == 0) s.n_cand = 0;
  __syncthreads();
  unsigned long long far_mass = 0;
  const auto place = [&](int v, float d, unsigned long long w) {
    if (d < kNearRange) {
      const int b = bucket_of(d);
      atomicAdd(&s.cnt0[b], 1u);
      atomicAdd(&s.mass[kBins + b], w);
      const uint32_t slot = atomicAdd(&s.n_cand, 1u);
      if (slot < (uint32_t)kSuperset) s.cand[slot] = key_from(d, v);
    } else {
      far_mass += w;
      if (use_k && d < kCountRange) atomicAdd(&s.cnt0[bucket_of(d)], 1u);
    }
  };
  if constexpr (QUAD) {
    // Nearly every quad lies outside the window and beyond the ranges that are bucketed: one
    // test each per quad, and the four weights are added without a branch.
    const float bucketed = use_k ? kCountRange : kNearRange;
    for_each_quad(c, [&](int v, const float4& z4, uint32_t word) {
      const float z[4] = {z4.x, z4.y, z4.z, z4.w};
      float d[4];
      unsigned long long w[4];
      if ((word >> (v & 28)) & 0xFu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) (void)key_of(c, v + e, z[e], word, &d[e]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) d[e] = plain_distance(c, z[e]);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = weight_of(d[e]);
      const float nearest = fminf(fminf(d[0], d[1]), fminf(d[2], d[3]));
      if (nearest < bucketed) {
#pragma unroll
        for (int e = 0; e < 4; ++e) place(v + e, d[e], w[e]);
      } else {
        far_mass += (w[0] + w[1]) + (w[2] + w[3]);
      }
    });
  } else {
    for_each_token(c, [&](int v, float z, uint32_t word) {
      float d;
      (void)key_of(c, v, z, word, &d);
      place(v, d, weight_of(d));
    });
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) far_mass += __shfl_xor(far_mass, o);
  if (lane == 0) s.wave_cnt[wv] = far_mass;
  __syncthreads();
  far_mass = 0;
  for (int k = 0; k < kWaves; ++k) far_mass += s.wave_cnt[k];
  uint32_t n_near = s.n_cand;
  __syncthreads();
  // the first cut that is needed: top-k by count, else top-p, else the draw itself, by weight
  scan_bins(s, s.cnt0, s.mass + kBins, count_buckets, false,
            greedy ? 1ull : use_k ? (unsigned long long)prm.top_k : ~0ull);
  int last_bucket = s.bin;
  const unsigned long long n_sup = last_bucket >= 0 ? s.before_cnt + s.cnt0[last_bucket] : 0;
  bool fast = n_near <= (uint32_t)kSuperset &&
              (!(greedy || use_k) || (last_bucket >= 0 && n_sup <= (unsigned long long)kSuperset));
  const unsigned long long all_mass = s.total_mass + far_mass;  // the whole vocabulary
  __syncthreads();
  if (fast && !greedy && !use_k) {
    unsigned long long thr;
    if (use_p) {
      thr = (unsigned long long)((double)prm.top_p * (double)all_mass);
      if (thr < 1) thr = 1;
    } else {
      thr = (unsigned long long)((double)u * (double)all_mass) + 1;
    }
    scan_bins(s, s.cnt0, s.mass + kBins, kNearBuckets, true, thr);
    fast = s.bin >= 0;
    last_bucket = s.bin;
    __syncthreads();
  }
  if (fast && last_bucket >= kNearBuckets) {
    // the k-th token lies beyond the near range: one more pass adds the tokens between the
    // near range and its bucket to the candidates
    for_each_token(c, [&](int v, float z, uint32_t word) {
      float d;
      const uint64_t comp = key_of(c, v, z, word, &d);
      if (d >= kNearRange && d < kCountRange && bucket_of(d) <= last_bucket)
        s.cand[atomicAdd(&s.n_cand, 1u)] = comp;
    });
    __syncthreads();
    n_near = s.n_cand;  // = n_sup
    __syncthreads();
  }

  int token = 0, n_kept = 1;
  if (!fast) {
    const Picked g = sample_general(s, c, prm.top_p, prm.top_k, greedy, u);
    token = g.token;
    n_kept = g.n_kept;
  } else {
    // keep the tokens up to the first cut's bucket (all later cuts lie among them), pad to a
    // power of two, sort by key; the histogram array is free now and takes the kept keys
    unsigned long long* keys = s.mass;
    if (tid == 0) s.n_cand = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n_near; i += kThreads) {
      const unsigned long long comp = s.cand[i];
      if (bucket_of(d_of_key(comp)) <= last_bucket) keys[atomicAdd(&s.n_cand, 1u)] = comp;
    }
    __syncthreads();
    const int m = (int)s.n_cand;
    if (m <= kThreads) {
      // few keys (the usual case under a top-k cut): a thread's key goes where the number of
      // smaller keys says (keys are distinct), two barriers instead of a sorting network's dozens
      const unsigned long long mine = tid < m ? keys[tid] : 0ull;
      int rank = 0;
      for (int j = 0; j < m; ++j) rank += keys[j] < mine ? 1 : 0;
      __syncthreads();
      if (tid < m) keys[rank] = mine;
      __syncthreads();
    }
    int np2 = 64;
    while (np2 < m) np2 <<= 1;
    if (m > kThreads) {
      for (int i = m + tid; i < np2; i += kThreads) keys[i] = ~0ull;
      __syncthreads();
    }
    for (int k = 2; m > kThreads && k <= np2; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int t = tid; t < np2 / 2; t += kThreads) {
          const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));  // lower index of the pair
          const int p = i | j;
          const bool up = (i & k) == 0;
          const unsigned long long x = keys[i], y = keys[p];
          if ((x > y) == up) {
            keys[i] = y;
            keys[p] = x;
          }
        }
        __syncthreads();
      }
    }
    // running sums of the sorted weights, in the candidate array (its keys were moved)
    unsigned long long* cum = s.cand;
    constexpr int kPer = kSuperset / kThreads;  // 4 consecutive entries per thread
    unsigned long long w4[kPer], run = 0;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int i = tid * kPer + e;
      w4[e] = i < m ? weight_of(d_of_key(keys[i])) : 0;
      run += w4[e];
    }
    unsigned long long inc = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned long long a = __shfl_up(inc, o);
      if (lane >= o) inc += a;
    }
    if (lane == 63) s.wave_mass[wv] = inc;
    __syncthreads();
    unsigned long long base = inc - run;
    for (int k = 0; k < wv; ++k) base += s.wave_mass[k];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      base += w4[e];
      cum[tid * kPer + e] = base;
    }
    __syncthreads();
    if (tid == 0) {
      if (greedy) {
        token = (int)(keys[0] & (kMaxVocab - 1));
        n_kept = 1;
      } else {
        unsigned long long total = all_mass;
        long long n = V;
        if (use_k) {  // top_k <= m: the count crossing was found among the near tokens
          n = prm.top_k;
          total = cum[prm.top_k - 1];
        }
        if (use_p) {
          unsigned long long thr = (unsigned long long)((double)prm.top_p * (double)total);
          if (thr < 1) thr = 1;
          const int j = first_reaching(cum, m, thr);  // < m: the crossing is among the near tokens
          n = j + 1;
          total = cum[j];
        }
        const unsigned long long target = (unsigned long long)((double)u * (double)total);
        const int i = first_reaching(cum, m, target + 1);
        token = (int)(keys[i] & (kMaxVocab - 1));
        n_kept = (int)n;
      }
    }
  }
  if (tid == 0) {
    tokens[stream] = token;
    if (kept) kept[stream] = n_kept;
  }
}

};  // Sampler

template <class Cfg>
__global__ __launch_bounds__(Cfg::kThreads) void sample_weights_kernel(
    int V, const float* __restrict__ logits, const vox_sampling_t* __restrict__ params,
    const int32_t* __restrict__ history, int window, float* __restrict__ d_out,
    unsigned long long* __restrict__ w_out) {
  Sampler<Cfg>::weights_body(V, logits, params, history, window, d_out, w_out);
}

template <class Cfg, bool QUAD>
__global__ __launch_bounds__(Cfg::kThreads, 4) void sample_kernel(
    int V, const float* __restrict__ logits, const vox_sampling_t* __restrict__ params,
    const int32_t* __restrict__ history, int window, const float* __restrict__ uniforms,
    int32_t* __restrict__ tokens, int32_t* __restrict__ kept) {
  Sampler<Cfg>::template sample_body<QUAD>(V, logits, params, history, window, uniforms, tokens,
                                           kept);
}

}  // namespace
}  // namespace vox

extern "C" int vox_sample(int32_t num_streams, int32_t vocab, const float* logits,
                          const vox_sampling_t* params, const int32_t* history, int32_t window,
                          const float* uniforms, int32_t* tokens, int32_t* kept,
                          void* hip_stream) {
  if (num_streams <= 0 || vocab <= 0 || vocab > vox::kMaxVocab || window < 0)
    return VOX_ERR_SHAPE;
  if (!logits || !params || !uniforms || !tokens || (window > 0 && !history)) return VOX_ERR_NULL;
  using namespace vox;
  const dim3 grid((unsigned)num_streams);
  hipStream_t st = (hipStream_t)hip_stream;
  // rows that start 16-byte aligned are read four tokens per lane and load
  const bool quad = vocab % 4 == 0 && ((uintptr_t)logits & 15) == 0;
  if (vocab <= SmallVocab::kVocab && quad)
    hipLaunchKernelGGL((sample_kernel<SmallVocab, true>), grid, dim3(SmallVocab::kThreads), 0, st,
                       vocab, logits, params, history, window, uniforms, tokens, kept);
  else if (vocab <= SmallVocab::kVocab)
    hipLaunchKernelGGL((sample_kernel<SmallVocab, false>), grid, dim3(SmallVocab::kThreads), 0, st,
                       vocab, logits, params, history, window, uniforms, tokens, kept);
  else if (quad)
    hipLaunchKernelGGL((sample_kernel<AnyVocab, true>), grid, dim3(AnyVocab::kThreads), 0, st,
                       vocab, logits, params, history, window, uniforms, tokens, kept);
  else
    hipLaunchKernelGGL((sample_kernel<AnyVocab, false>), grid, dim3(AnyVocab::kThreads), 0, st,
                       vocab, logits, params, history, window, uniforms, tokens, kept);
  return hipGetLastError() == hipSuccess ? VOX_OK : VOX_ERR_HIP;
}

extern "C" int vox_sample_weights(int32_t num_streams, int32_t vocab, const float* logits,
                                  const vox_sampling_t* params, const int32_t* history,
                                  int32_t window, float* d_out, uint64_t* w_out,
                                  void* hip_stream) {
  if (num_streams <= 0 || vocab <= 0 || vocab > vox::kMaxVocab || window < 0)
    return VOX_ERR_SHAPE;
  if (!logits || !params || !d_out || !w_out || (window > 0 && !history)) return VOX_ERR_NULL;
  hipLaunchKernelGGL(vox::sample_weights_kernel<vox::AnyVocab>, dim3((unsigned)num_streams),
                     dim3(vox::AnyVocab::kThreads), 0, (hipStream_t)hip_stream, vocab, logits,
                     params, history, window, d_out, (unsigned long long*)w_out);
  return hipGetLastError() == hipSuccess ? VOX_OK : VOX_ERR_HIP;
}
