// KV append, block gather, split-K planning and the partial-softmax merge.
#include "vox_common.hpp"

namespace vox {
namespace {

// ---------------------------------------------------------------------------------------
// KV append: one thread per (stream, kv head, 8-dim slice).  The K slice of one token is a
// contiguous 16 bytes in the K pool; the V slice is eight 2-byte slots 32 bytes apart.
__global__ __launch_bounds__(256) void kv_append_kernel(Params p, const uint4* __restrict__ k_new,
                                                        const uint4* __restrict__ v_new,
                                                        uint16_t* __restrict__ k_pool,
                                                        uint16_t* __restrict__ v_pool,
                                                        const int32_t* __restrict__ bt,
                                                        const int32_t* __restrict__ lens) {
  const int slices = p.D >> 3;
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= (int64_t)p.S * p.Hkv * slices) return;
  const int o = (int)(x % slices);
  const int h = (int)((x / slices) % p.Hkv);
  const int s = (int)(x / ((int64_t)slices * p.Hkv));
  const int L = lens[s];
  if (L <= 0) return;
  const int pos = L - 1;
  const int64_t blk = bt[(int64_t)s * p.max_nb + (pos >> 4)];
  const int t = pos & (kBlock - 1);
  const size_t g = granule_offset(blk, h, p.Hkv, p.D);
  const uint4 kv = k_new[x];
  *reinterpret_cast<uint4*>(k_pool + g + k_elem(t, o * 8)) = kv;
  const uint4 vv = v_new[x];
  const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint16_t bits = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
    v_pool[g + v_elem(t, o * 8 + e)] = bits;
  }
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
      const uint32_t lo = v_pool[g + v_elem(t, o * 8 + e)];
      const uint32_t hi = v_pool[g + v_elem(t, o * 8 + e + 1)];
      w[e >> 1] = lo | (hi << 16);
    }
    v_out[dst] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// ---------------------------------------------------------------------------------------
// Plan: per stream, n = ceil(nb / chunk) items of equal even length ceil(nb / n) rounded up to
// a multiple of two blocks (the last item takes the remainder).  One workgroup; streams are
// scanned 1024 at a time.
__global__ __launch_bounds__(1024) void plan_kernel(const int32_t* __restrict__ lens, int S,
                                                    int chunk, int capacity,
                                                    int32_t* __restrict__ header,
                                                    int32_t* __restrict__ first_item,
                                                    Item* __restrict__ items) {
  __shared__ int scan[1024];
  __shared__ int carry;
  __shared__ int overflow;
  const int tid = threadIdx.x;
  if (tid == 0) {
    carry = 0;
    overflow = 0;
  }
  __syncthreads();
  for (int base = 0; base < S; base += 1024) {
    const int s = base + tid;
    int nb = 0, n = 0, len = 0;
    if (s < S) {
      const int L = lens[s];
      nb = L > 0 ? (L + kBlock - 1) / kBlock : 0;
      n = (nb + chunk - 1) / chunk;
      if (n) len = (((nb + n - 1) / n) + 1) & ~1;
    }
    scan[tid] = n;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const int v = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += v;
      __syncthreads();
    }
    const int first = carry + scan[tid] - n;
    if (s < S) {
      first_item[s] = min(first, capacity);
      for (int c = 0; c < n; ++c) {
        const int idx = first + c;
        if (idx < capacity) {
          Item it;
          it.stream = s;
          it.first_block = c * len;
          it.nblocks = min(len, nb - c * len);
          it.pad = 0;
          items[idx] = it;
        } else {
          overflow = 1;
        }
      }
    }
    __syncthreads();
    if (tid == 1023) carry += scan[1023];
    __syncthreads();
  }
  if (tid == 0) {
    first_item[S] = min(carry, capacity);
    header[0] = min(carry, capacity);
    header[1] = chunk;
    header[2] = overflow;
  }
}

// ---------------------------------------------------------------------------------------
// Merge: one wave per (stream, q head).  Lanes hold the chunks' (max, sum) records; the global
// max and the rescaled sum are wave reductions; the accumulators are then combined with each
// lane owning D/64 output dims.
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

template <int D>
__global__ __launch_bounds__(256) void merge_kernel(Params p, const int32_t* __restrict__ first_item,
                                                    const float2* __restrict__ pml,
                                                    const float* __restrict__ pacc,
                                                    float* __restrict__ out,
                                                    float* __restrict__ lse) {
  constexpr int DPL = D / kWave;  // dims per lane
  const int lane = threadIdx.x & (kWave - 1);
  const int w = blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);
  if (w >= p.S * p.Hq) return;
  const int s = w / p.Hq, i = w % p.Hq;
  const int f0 = first_item[s];
  const int n = first_item[s + 1] - f0;
  float m_run = -INFINITY, l_run = 0.f;
  float acc[DPL];
#pragma unroll
  for (int k = 0; k < DPL; ++k) acc[k] = 0.f;
  for (int c0 = 0; c0 < n; c0 += kWave) {
    const int c = c0 + lane;
    float2 ml = make_float2(-INFINITY, 0.f);
    if (c < n) ml = pml[(size_t)(f0 + c) * p.Hq + i];
    const float m_new = fmaxf(m_run, wave_max(ml.x));
    const float wgt = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - m_new);
    const float alpha = (m_run == -INFINITY) ? 0.f : exp2f(m_run - m_new);
    l_run = l_run * alpha + wave_sum(wgt * ml.y);
#pragma unroll
    for (int k = 0; k < DPL; ++k) acc[k] *= alpha;
    const int cnt = min(kWave, n - c0);
    for (int j = 0; j < cnt; ++j) {
      const float wj = __shfl(wgt, j);
      const float* src = pacc + ((size_t)(f0 + c0 + j) * p.Hq + i) * D + lane * DPL;
      if (DPL == 2) {
        const float2 a = *reinterpret_cast<const float2*>(src);
        acc[0] += wj * a.x;
        acc[DPL - 1] += wj * a.y;
      } else {
        acc[0] += wj * src[0];
      }
    }
    m_run = m_new;
  }
  float* dst = out + ((size_t)s * p.Hq + i) * D + lane * DPL;
  const float inv = (n > 0 && l_run > 0.f) ? 1.f / l_run : 0.f;
#pragma unroll
  for (int k = 0; k < DPL; ++k) dst[k] = acc[k] * inv;
  if (lse && lane == 0)
    lse[(size_t)s * p.Hq + i] =
        (n > 0 && l_run > 0.f) ? (m_run + log2f(l_run)) * 0.69314718055994530942f : -INFINITY;
}

}  // namespace

hipError_t launch_kv_append(const Params& p, const void* k_new, const void* v_new, void* k_pool,
                            void* v_pool, const int32_t* bt, const int32_t* lens,
                            hipStream_t st) {
  const int64_t n = (int64_t)p.S * p.Hkv * (p.D / 8);
  const unsigned grid = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(kv_append_kernel, dim3(grid), dim3(256), 0, st, p, (const uint4*)k_new,
                     (const uint4*)v_new, (uint16_t*)k_pool, (uint16_t*)v_pool, bt, lens);
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

hipError_t launch_plan(const Params& p, const int32_t* lens, int chunk_blocks, int capacity,
                       int32_t* header, int32_t* first_item, Item* items, hipStream_t st) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(1024), 0, st, lens, p.S, chunk_blocks, capacity,
                     header, first_item, items);
  return hipGetLastError();
}

hipError_t launch_merge(const Params& p, const int32_t* first_item, const float2* partial_ml,
                        const float* partial_acc, float* out, float* lse, hipStream_t st) {
  const unsigned grid = (unsigned)(((int64_t)p.S * p.Hq + kWavesPerGroup - 1) / kWavesPerGroup);
  if (p.D == 128)
    hipLaunchKernelGGL(merge_kernel<128>, dim3(grid), dim3(256), 0, st, p, first_item, partial_ml,
                       partial_acc, out, lse);
  else
    hipLaunchKernelGGL(merge_kernel<64>, dim3(grid), dim3(256), 0, st, p, first_item, partial_ml,
                       partial_acc, out, lse);
  return hipGetLastError();
}

}  // namespace vox
