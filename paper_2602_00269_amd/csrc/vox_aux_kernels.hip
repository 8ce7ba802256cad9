// KV append, block gather, split-K planning and the partial-softmax merge.
#include "vox_merge.hpp"

namespace vox {
namespace {

// ---------------------------------------------------------------------------------------
// KV append: one wave per (stream, kv head).  The token's K row is D/32 pieces of 64 bytes:
// lanes [0, D/8) each copy 16 bytes.  Its V row is one 2-byte slot in each 8-byte token quad
// of a D*8-byte region; lanes [0, D/2) read the 16 bytes holding two dims of that region,
// replace the token's two slots and store the 16 bytes back, so the region's D/16 cache lines
// are written whole.  Lines that were just written are slow for the following attention
// kernel to read, so the layout keeps their number small (D/32 + D/16 per kv head).
typedef uint32_t au32x4 __attribute__((ext_vector_type(4)));

// V row of token t into its block: lanes [0, D/2) rewrite the 16 bytes that hold their two dims.
template <int D>
__device__ inline void insert_v(uint16_t* __restrict__ v_pool, size_t g, int t, int lane,
                                const uint16_t* __restrict__ vrow) {
  if (lane < D / 2) {
    uint16_t* quad = v_pool + g + v_elem(t & ~3, 2 * lane, D);  // dims 2*lane, 2*lane+1
    au32x4 r = *reinterpret_cast<const au32x4*>(quad);
    const uint32_t two = *reinterpret_cast<const uint32_t*>(vrow + 2 * lane);
    const int e = t & 3;  // slot of the token inside each 4-token quad
    const uint32_t d0 = two & 0xFFFFu, d1 = two >> 16;
    const uint32_t keep = (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
    const int sh = (e & 1) * 16;
    r[e >> 1] = (r[e >> 1] & keep) | (d0 << sh);
    r[2 + (e >> 1)] = (r[2 + (e >> 1)] & keep) | (d1 << sh);
    *reinterpret_cast<au32x4*>(quad) = r;
  }
}

template <int D>
__device__ inline void append_role(const Params& p, int group, const uint16_t* __restrict__ k_new,
                                   const uint16_t* __restrict__ v_new,
                                   uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool,
                                   const int32_t* __restrict__ bt,
                                   const int32_t* __restrict__ lens) {
  const int lane = threadIdx.x & (kWave - 1);
  const int sigma = group * kWavesPerGroup + (threadIdx.x >> 6);
  if (sigma >= p.S * p.Hkv) return;
  const int s = sigma / p.Hkv, h = sigma % p.Hkv;
  const int L = lens[s];
  if (L <= 0) return;
  const int pos = L - 1;
  const int64_t blk = bt[(int64_t)s * p.max_nb + (pos >> 4)];
  const int t = pos & (kBlock - 1);
  const size_t g = granule_offset(blk, h, p.Hkv, D);
  const uint16_t* krow = k_new + (size_t)sigma * D;
  const uint16_t* vrow = v_new + (size_t)sigma * D;
  if (lane < D / 8)
    *reinterpret_cast<au32x4*>(k_pool + g + k_elem(t, lane * 8)) =
        *reinterpret_cast<const au32x4*>(krow + lane * 8);
  insert_v<D>(v_pool, g, t, lane, vrow);
}

// Fused-mode append: one wave per (stream, q head or kv head).  Lane j < D/4 owns the rotation
// pairs (i, i + D/2) for i = 2j, 2j+1.  The arithmetic is fixed, because it decides bf16 codes:
// two fp32 products and their sum or difference as separate roundings (contraction is off in
// this function), then round-to-nearest-even to bf16 done on the bits.
__device__ inline uint32_t bf16_rne_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (u >> 16) | 0x0040u;  // NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ inline float bf16_bits_to_f32(uint32_t b) { return __builtin_bit_cast(float, b << 16); }

template <int D>
__device__ inline void rope_append_role(const Params& p, int group, const AppendArgs& a,
                                        const int32_t* __restrict__ bt,
                                        const int32_t* __restrict__ lens) {
#pragma clang fp contract(off)
  const int lane = threadIdx.x & (kWave - 1);
  const int x = group * kWavesPerGroup + (threadIdx.x >> 6);
  const int slots = p.Hq + p.Hkv;
  if (x >= p.S * slots) return;
  const int s = x / slots, hs = x % slots;
  const int L = lens[s];
  if (L <= 0) return;
  const int pos = L - 1;
  const uint16_t* row = a.qkv + ((size_t)s * (p.Hq + 2 * p.Hkv) + hs) * D;  // q heads, then k heads
  uint32_t lo = 0, hi = 0;
  if (lane < D / 4) {
    const uint32_t x1 = *reinterpret_cast<const uint32_t*>(row + 2 * lane);
    const uint32_t x2 = *reinterpret_cast<const uint32_t*>(row + D / 2 + 2 * lane);
    const float2 c = *reinterpret_cast<const float2*>(a.rope_cos + (size_t)pos * (D / 2) + 2 * lane);
    const float2 sn = *reinterpret_cast<const float2*>(a.rope_sin + (size_t)pos * (D / 2) + 2 * lane);
    const float a0 = bf16_bits_to_f32(x1 & 0xFFFFu), a1 = bf16_bits_to_f32(x1 >> 16);
    const float b0 = bf16_bits_to_f32(x2 & 0xFFFFu), b1 = bf16_bits_to_f32(x2 >> 16);
    const float a0c = a0 * c.x, b0s = b0 * sn.x, b0c = b0 * c.x, a0s = a0 * sn.x;
    const float a1c = a1 * c.y, b1s = b1 * sn.y, b1c = b1 * c.y, a1s = a1 * sn.y;
    lo = bf16_rne_bits(a0c - b0s) | (bf16_rne_bits(a1c - b1s) << 16);
    hi = bf16_rne_bits(b0c + a0s) | (bf16_rne_bits(b1c + a1s) << 16);
  }
  if (hs < p.Hq) {
    if (lane < D / 4) {
      uint16_t* dst = a.q_out + ((size_t)s * p.Hq + hs) * D;
      *reinterpret_cast<uint32_t*>(dst + 2 * lane) = lo;
      *reinterpret_cast<uint32_t*>(dst + D / 2 + 2 * lane) = hi;
    }
    return;
  }
  const int h = hs - p.Hq;
  const int64_t blk = bt[(int64_t)s * p.max_nb + (pos >> 4)];
  const int t = pos & (kBlock - 1);
  const size_t g = granule_offset(blk, h, p.Hkv, D);
  if (lane < D / 4) {
    *reinterpret_cast<uint32_t*>(a.k_pool + g + k_elem(t, 2 * lane)) = lo;
    *reinterpret_cast<uint32_t*>(a.k_pool + g + k_elem(t, D / 2 + 2 * lane)) = hi;
  }
  insert_v<D>(a.v_pool, g, t, lane, row + (size_t)p.Hkv * D);  // v head h follows the k heads
}

// Either mode of the append, by what the arguments carry.
template <int D>
__device__ inline void any_append_role(const Params& p, int group, const AppendArgs& a,
                                       const int32_t* __restrict__ bt,
                                       const int32_t* __restrict__ lens) {
  if (a.qkv)
    rope_append_role<D>(p, group, a, bt, lens);
  else
    append_role<D>(p, group, a.k_new, a.v_new, a.k_pool, a.v_pool, bt, lens);
}

template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(Params p, AppendArgs a,
                                                        const int32_t* __restrict__ bt,
                                                        const int32_t* __restrict__ lens) {
  any_append_role<D>(p, blockIdx.x, a, bt, lens);
}

// ---------------------------------------------------------------------------------------
// Gather: workgroup (x = stream, y = 64-token window); thread per (token, head, 8-dim slice).
constexpr int kGatherTokens = 64;

__global__ __launch_bounds__(256) void kv_gather_kernel(Params p, const uint16_t* __restrict__ k_pool,
                                                        const uint16_t* __restrict__ v_pool,
                                                        const int32_t* __restrict__ bt,
                                                        const int32_t* __restrict__ lens,
                                                        const int64_t* __restrict__ row_offsets,
                                                        uint4* __restrict__ k_out,
                                                        uint4* __restrict__ v_out) {
  const int s = blockIdx.x;
  const int L = lens[s];
  const int t0 = blockIdx.y * kGatherTokens;
  if (t0 >= L) return;
  const int t1 = min(L, t0 + kGatherTokens);
  const int slices = p.D >> 3;
  const int per_token = p.Hkv * slices;
  const int64_t row0 = row_offsets[s];
  for (int x = threadIdx.x; x < (t1 - t0) * per_token; x += blockDim.x) {
    const int tok = t0 + x / per_token;
    const int h = (x % per_token) / slices;
    const int o = x % slices;
    const int64_t blk = bt[(int64_t)s * p.max_nb + (tok >> 4)];
    const int t = tok & (kBlock - 1);
    const size_t g = granule_offset(blk, h, p.Hkv, p.D);
    const size_t dst = ((size_t)(row0 + tok) * p.Hkv + h) * slices + o;
    k_out[dst] = *reinterpret_cast<const uint4*>(k_pool + g + k_elem(t, o * 8));
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const uint32_t lo = v_pool[g + v_elem(t, o * 8 + e, p.D)];
      const uint32_t hi = v_pool[g + v_elem(t, o * 8 + e + 1, p.D)];
      w[e >> 1] = lo | (hi << 16);
    }
    v_out[dst] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// ---------------------------------------------------------------------------------------
// Plan: writes the step prefix, the header (N, Q, W) and one descriptor per global step.
// Every workgroup rebuilds the exclusive scan of n_s = ceil(ceil(L_s/16)/2) in LDS (S is
// small: a slice per thread, a shuffle scan per wave, one pass over the wave totals), then
// each thread expands one global step: binary search for the stream, then head and step
// inside the segment.  Workgroup 0 also publishes the scan.
constexpr int kPlanThreads = 256;
constexpr int kPlanMaxStreams = kMaxStreams;  // LDS-resident prefix

__device__ inline void plan_role(const Params& p, int group, const int32_t* __restrict__ bt,
                                 const int32_t* __restrict__ lens, int waves,
                                 int64_t desc_capacity, int32_t* __restrict__ header,
                                 int32_t* __restrict__ step_prefix, int4* __restrict__ desc) {
  __shared__ int prefix[kPlanMaxStreams + 1];
  __shared__ int wave_total[kPlanThreads / kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const int S = p.S;
  const int per = (S + kPlanThreads - 1) / kPlanThreads;
  const int lo = min(S, tid * per), hi = min(S, lo + per);
  int run = 0;
  for (int s = lo; s < hi; ++s) {
    const int L = lens[s];
    const int nb = L > 0 ? (L + kBlock - 1) / kBlock : 0;
    prefix[s] = run;  // exclusive inside the slice
    run += (nb + 1) >> 1;
  }
  int incl = run;  // inclusive scan of the slice totals inside the wave
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == kWave - 1) wave_total[wv] = incl;
  __syncthreads();
  int before = incl - run;
  for (int k = 0; k < wv; ++k) before += wave_total[k];
  for (int s = lo; s < hi; ++s) prefix[s] += before;
  if (tid == kPlanThreads - 1) prefix[S] = before + run;
  __syncthreads();

  const int64_t n_all = (int64_t)prefix[S] * p.Hkv;
  const int64_t N = min(n_all, desc_capacity);
  const StepLayout lay = layout_of(N, waves, p.pool_counter != nullptr);
  if (group == 0) {
    for (int s = tid; s <= S; s += kPlanThreads) step_prefix[s] = prefix[s];
    for (int l = tid; l < kMaxLayers; l += kPlanThreads) header[kHdrPoolCounters + l] = 0;
    if (tid == 0) {
      header[kHdrSteps] = (int)N;
      header[kHdrPerWave] = lay.Q;
      header[kHdrWaves] = waves;
      header[kHdrOverflow] = n_all > desc_capacity;
      header[kHdrMain] = (int)lay.n_main;
      header[kHdrUsed] = lay.U;
      header[kHdrPool] = lay.R;
    }
  }

  const int64_t x = (int64_t)group * kPlanThreads + tid;
  if (x >= N) return;
  // largest s with Hkv * prefix[s] <= x (streams with n_s == 0 share a prefix and are skipped)
  int a = 0, b = S;
  while (b - a > 1) {
    const int mid = (a + b) >> 1;
    if ((int64_t)prefix[mid] * p.Hkv <= x)
      a = mid;
    else
      b = mid;
  }
  const int s = a;
  const int n = prefix[s + 1] - prefix[s];
  const int r = (int)(x - (int64_t)prefix[s] * p.Hkv);
  const int h = r / n, st = r - h * n;
  const int L = lens[s];
  const int nb = (L + kBlock - 1) / kBlock;
  const int32_t* row = bt + (size_t)s * p.max_nb;
  const int ida = row[2 * st];
  const int idb = (2 * st + 1 < nb) ? row[2 * st + 1] : ida;
  const int ntok = min(kStepTokens, L - kStepTokens * st);
  int meta = ntok;
  if (st == 0 || step_opens_range(lay, x)) meta |= kMetaFirst;
  if (st == n - 1 || step_closes_range(lay, x)) meta |= kMetaLast;
  if (st == n - 1) meta |= kMetaTail;
  desc[x] = make_int4(ida * p.Hkv + h, idb * p.Hkv + h, meta, s * p.Hkv + h);
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(
    Params p, const int32_t* __restrict__ bt, const int32_t* __restrict__ lens, int waves,
    int64_t desc_capacity, int32_t* __restrict__ header, int32_t* __restrict__ step_prefix,
    int4* __restrict__ desc) {
  plan_role(p, blockIdx.x, bt, lens, waves, desc_capacity, header, step_prefix, desc);
}

// Plan and the first layer's append in one launch: the two are independent and both are
// short chains of dependent loads, so running them side by side hides one behind the other.
template <int D>
__global__ __launch_bounds__(kPlanThreads) void plan_append_kernel(
    Params p, int plan_groups, AppendArgs a, const int32_t* __restrict__ bt,
    const int32_t* __restrict__ lens, int waves, int64_t desc_capacity,
    int32_t* __restrict__ header, int32_t* __restrict__ step_prefix, int4* __restrict__ desc) {
  if ((int)blockIdx.x < plan_groups)
    plan_role(p, blockIdx.x, bt, lens, waves, desc_capacity, header, step_prefix, desc);
  else
    any_append_role<D>(p, blockIdx.x - plan_groups, a, bt, lens);
}

// ---------------------------------------------------------------------------------------
// Merge: one wave per (stream, q head).  The runs of segment sigma lie in the ranges r0 .. r1 of
// its first and last global step; run j is slot r0 + j + sigma.
// Lanes hold the runs' (max, sum) records; the global max and the rescaled sum are wave
// reductions; the accumulators are then combined with each lane owning D/64 output dims.
template <int D>
__device__ inline void merge_role(const Params& p, int group, const int32_t* __restrict__ header,
                                  const int32_t* __restrict__ step_prefix,
                                  const float2* __restrict__ pml, const float* __restrict__ pacc,
                                  float* __restrict__ out, float* __restrict__ lse) {
  const int lane = threadIdx.x & (kWave - 1);
  const int w = group * kWavesPerGroup + (threadIdx.x >> 6);
  if (w >= p.S * p.Hq) return;
  const int s = w / p.Hq, i = w % p.Hq;
  const int h = i / p.G, g = i % p.G;
  const int sigma = s * p.Hkv + h;
  const StepLayout lay = p.n_steps >= 0 ? p.lay : layout_from_header(header);
  const int64_t N = lay.N;
  const int nseg = step_prefix[s + 1] - step_prefix[s];
  const int64_t first = (int64_t)step_prefix[s] * p.Hkv + (int64_t)h * nseg;
  int n = 0;          // number of runs
  int64_t slot0 = 0;  // slot of run 0
  if (nseg > 0 && first < N) {
    const int64_t last = min(N, first + nseg) - 1;
    const int64_t r0 = range_of_step(lay, first), r1 = range_of_step(lay, last);
    n = (int)(r1 - r0 + 1);
    slot0 = r0 + sigma;
  }
  if (p.q_rows && n == 0) return;  // packed rows: a stream without a run owns no output row
  const size_t row = (size_t)(p.q_rows ? p.q_rows[s] : s) * p.Hq + i;
  merge_runs<D>(pml, pacc, slot0, n, p.G, g, lane, out + row * D, lse ? lse + row : nullptr);
}

template <int D>
__global__ __launch_bounds__(256) void merge_kernel(Params p, const int32_t* __restrict__ header,
                                                    const int32_t* __restrict__ step_prefix,
                                                    const float2* __restrict__ pml,
                                                    const float* __restrict__ pacc,
                                                    float* __restrict__ out,
                                                    float* __restrict__ lse) {
  merge_role<D>(p, blockIdx.x, header, step_prefix, pml, pacc, out, lse);
}

// Merge of layer l and the append of layer l + 1 in one launch (independent buffers).
template <int D>
__global__ __launch_bounds__(256) void merge_append_kernel(
    Params p, int merge_grps, const int32_t* __restrict__ header,
    const int32_t* __restrict__ step_prefix, const float2* __restrict__ pml,
    const float* __restrict__ pacc, float* __restrict__ out, AppendArgs a,
    const int32_t* __restrict__ bt, const int32_t* __restrict__ lens) {
  if ((int)blockIdx.x < merge_grps)
    merge_role<D>(p, blockIdx.x, header, step_prefix, pml, pacc, out, nullptr);
  else
    any_append_role<D>(p, blockIdx.x - merge_grps, a, bt, lens);
}

// Streaming-read probe with the attention kernel's memory pipeline and none of its arithmetic:
// one wave per SIMD of the chip, each walks a contiguous share of the buffer in 16 KB steps
// (16 loads of 16 bytes per lane, every load instruction one contiguous KB) through a ring of
// three steps in flight, and only xors what arrives.  The buffer's tail that is no whole step
// is read by a plain strided loop.
constexpr int kProbeStepVecs = 1024;  // 16-byte vectors per step
constexpr int kProbeRing = 3;
constexpr int kProbeGroups = kDesignWaveSlots / kWavesPerGroup;

__global__ __launch_bounds__(256, 1) void read_probe_kernel(const au32x4* __restrict__ buf,
                                                            size_t vecs,
                                                            uint32_t* __restrict__ sink) {
  constexpr int kLoads = kProbeStepVecs / kWave;
  const int lane = threadIdx.x & (kWave - 1);
  const size_t w = (size_t)blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);
  const size_t waves = (size_t)gridDim.x * kWavesPerGroup;
  const size_t steps = vecs / kProbeStepVecs;
  const size_t per = (steps + waves - 1) / waves;
  const size_t s0 = min(steps, w * per), s1 = min(steps, s0 + per);
  const long long n = (long long)(s1 - s0);
  const au32x4* base = buf + s0 * kProbeStepVecs + lane;
  au32x4 acc = {0, 0, 0, 0};
  au32x4 ring[kProbeRing][kLoads];
  // refills past the share's end re-read its first step (in range, cache resident) and are
  // dropped, so that the steady loop carries no condition around its loads
#define VOX_PROBE_FILL(B, I)                                                          \
  {                                                                                   \
    const au32x4* src = base + ((I) < n ? (size_t)(I) : 0) * kProbeStepVecs;           \
    _Pragma("unroll") for (int j = 0; j < kLoads; ++j) ring[B][j] =                    \
        __builtin_nontemporal_load(src + j * kWave);                                  \
  }
  if (n > 0) {
#pragma unroll
    for (int b = 0; b < kProbeRing; ++b) VOX_PROBE_FILL(b, b)
    for (long long i0 = 0; i0 < n; i0 += kProbeRing) {
#pragma unroll
      for (int b = 0; b < kProbeRing; ++b) {
        if (i0 + b < n) {
#pragma unroll
          for (int j = 0; j < kLoads; ++j) acc ^= ring[b][j];
        }
        VOX_PROBE_FILL(b, i0 + b + kProbeRing)
      }
    }
  }
#undef VOX_PROBE_FILL
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = steps * kProbeStepVecs + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < vecs;
       i += stride)
    acc ^= __builtin_nontemporal_load(buf + i);
  uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
  if (lane == 0) atomicXor(&sink[blockIdx.x], x);
}

}  // namespace

static unsigned host_append_groups(const Params& p, const AppendArgs& a) {
  const int64_t waves = (int64_t)p.S * (a.qkv ? p.Hq + p.Hkv : p.Hkv);
  return (unsigned)((waves + kWavesPerGroup - 1) / kWavesPerGroup);
}
static unsigned host_merge_groups(const Params& p) {
  return (unsigned)(((int64_t)p.S * p.Hq + kWavesPerGroup - 1) / kWavesPerGroup);
}
static unsigned host_plan_groups(int64_t max_steps) {
  return (unsigned)max((int64_t)1, (max_steps + kPlanThreads - 1) / kPlanThreads);
}

hipError_t launch_append(const Params& p, const AppendArgs& a, const int32_t* bt,
                         const int32_t* lens, hipStream_t st) {
  if (p.D == 128)
    hipLaunchKernelGGL(kv_append_kernel<128>, dim3(host_append_groups(p, a)), dim3(256), 0, st, p,
                       a, bt, lens);
  else
    hipLaunchKernelGGL(kv_append_kernel<64>, dim3(host_append_groups(p, a)), dim3(256), 0, st, p,
                       a, bt, lens);
  return hipGetLastError();
}

hipError_t launch_kv_gather(const Params& p, const void* k_pool, const void* v_pool,
                            const int32_t* bt, const int32_t* lens, const int64_t* row_offsets,
                            void* k_out, void* v_out, hipStream_t st) {
  const unsigned windows =
      (unsigned)(((int64_t)p.max_nb * kBlock + kGatherTokens - 1) / kGatherTokens);
  hipLaunchKernelGGL(kv_gather_kernel, dim3(p.S, windows), dim3(256), 0, st, p,
                     (const uint16_t*)k_pool, (const uint16_t*)v_pool, bt, lens, row_offsets,
                     (uint4*)k_out, (uint4*)v_out);
  return hipGetLastError();
}

hipError_t launch_plan(const Params& p, const int32_t* bt, const int32_t* lens, int waves,
                       int64_t desc_capacity, int64_t max_steps, int32_t* header,
                       int32_t* step_prefix, int4* desc, hipStream_t st) {
  if (p.S > kPlanMaxStreams) return hipErrorInvalidValue;
  hipLaunchKernelGGL(plan_kernel, dim3(host_plan_groups(max_steps)), dim3(kPlanThreads), 0, st, p,
                     bt, lens, waves, desc_capacity, header, step_prefix, desc);
  return hipGetLastError();
}

hipError_t launch_plan_append(const Params& p, const int32_t* bt, const int32_t* lens, int waves,
                              int64_t desc_capacity, int64_t max_steps, int32_t* header,
                              int32_t* step_prefix, int4* desc, const AppendArgs& a,
                              hipStream_t st) {
  if (p.S > kPlanMaxStreams) return hipErrorInvalidValue;
  const unsigned pg = host_plan_groups(max_steps);
  if (p.D == 128)
    hipLaunchKernelGGL(plan_append_kernel<128>, dim3(pg + host_append_groups(p, a)),
                       dim3(kPlanThreads), 0, st, p, (int)pg, a, bt, lens, waves, desc_capacity,
                       header, step_prefix, desc);
  else
    hipLaunchKernelGGL(plan_append_kernel<64>, dim3(pg + host_append_groups(p, a)),
                       dim3(kPlanThreads), 0, st, p, (int)pg, a, bt, lens, waves, desc_capacity,
                       header, step_prefix, desc);
  return hipGetLastError();
}

hipError_t launch_merge(const Params& p, const int32_t* header, const int32_t* step_prefix,
                        const float2* partial_ml, const float* partial_acc, float* out,
                        float* lse, hipStream_t st) {
  if (p.D == 128)
    hipLaunchKernelGGL(merge_kernel<128>, dim3(host_merge_groups(p)), dim3(256), 0, st, p, header,
                       step_prefix, partial_ml, partial_acc, out, lse);
  else
    hipLaunchKernelGGL(merge_kernel<64>, dim3(host_merge_groups(p)), dim3(256), 0, st, p, header,
                       step_prefix, partial_ml, partial_acc, out, lse);
  return hipGetLastError();
}

hipError_t launch_merge_append(const Params& p, const int32_t* header, const int32_t* step_prefix,
                               const float2* partial_ml, const float* partial_acc, float* out,
                               const int32_t* bt, const int32_t* lens, const AppendArgs& a,
                               hipStream_t st) {
  const unsigned mg = host_merge_groups(p);
  if (p.D == 128)
    hipLaunchKernelGGL(merge_append_kernel<128>, dim3(mg + host_append_groups(p, a)), dim3(256), 0,
                       st, p, (int)mg, header, step_prefix, partial_ml, partial_acc, out, a, bt,
                       lens);
  else
    hipLaunchKernelGGL(merge_append_kernel<64>, dim3(mg + host_append_groups(p, a)), dim3(256), 0,
                       st, p, (int)mg, header, step_prefix, partial_ml, partial_acc, out, a, bt,
                       lens);
  return hipGetLastError();
}

hipError_t launch_read_probe(const void* buf, size_t bytes, void* sink, hipStream_t st) {
  hipLaunchKernelGGL(read_probe_kernel, dim3(kProbeGroups), dim3(256), 0, st, (const au32x4*)buf,
                     bytes / 16, (uint32_t*)sink);
  return hipGetLastError();
}

}  // namespace vox
