// Shared declarations of the HIP library: kernel parameter block, workspace map and the
// cache-layout index helpers.  gfx950 only.
//
// Split-K decomposition.  The context of stream s is walked in steps of 32 tokens (two KV
// blocks); n_s = ceil(ceil(L_s / 16) / 2).  Segment sigma = s * Hkv + h owns n_s steps.  All
// segments are laid end to end on one axis of N = Hkv * sum_s n_s global steps, and that axis
// is cut into ranges (StepLayout below): W equal ones, one per wave, and for long axes a pool
// of short ones that waves take as they finish.  A wave therefore starts with the same number
// of KV bytes as every other wave whatever the length mix, and a range may cover the tail of
// one segment, several whole short segments and the head of another.  Every maximal run of one
// segment inside one range yields one partial record (max, sum, accumulator); ranges and runs
// are numbered along the axis, so the record of the run of segment sigma in range r is slot
// r + sigma.  The merge kernel recomputes which ranges a segment crosses from the prefix sums
// and the layout alone.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vox.h"

namespace vox {

constexpr int kBlock = 16;         // tokens per KV block
constexpr int kWave = 64;          // lanes per wavefront
constexpr int kWavesPerGroup = 4;  // decode / merge workgroups are 4 independent waves
constexpr int kStepTokens = 32;    // tokens consumed per step (two blocks)
constexpr int kMaxStreams = 8192;  // the plan kernel keeps the per-stream prefix in LDS
constexpr int kDesignWaveSlots = 256 * kWavesPerGroup;  // 256 CUs x 1 workgroup x 4 waves (1 per SIMD)

// Step descriptor written by the plan kernels, one per global step (16 bytes).
//   x: granule index (block id * Hkv + h) of the step's first block
//   y: granule index of its second block (= x when the stream has no such block)
//   z: bits 0..5 valid tokens in the step (1..32), bit 8 first step of a run, bit 9 last,
//      bit 10 last step of the stream
//   w: segment index sigma
constexpr int kMetaFirst = 1 << 8;
constexpr int kMetaLast = 1 << 9;
constexpr int kMetaTail = 1 << 10;  // last step of its stream: holds the block appended to
// multi-token step, on a segment's last step: the whole segment is this one run, its rows go
// straight to the output
constexpr int kMetaWhole = 1 << 11;
constexpr int kMetaTokMask = 63;

// header words
constexpr int kHdrSteps = 0;     // N
constexpr int kHdrPerWave = 1;   // Q
constexpr int kHdrWaves = 2;     // W
constexpr int kHdrOverflow = 3;  // set when N exceeded the descriptor capacity
constexpr int kHdrMain = 4;      // n_main, U, R of the layout (see StepLayout)
constexpr int kHdrUsed = 5;
constexpr int kHdrPool = 6;
constexpr int kHdrPoolCounters = 64;  // one pool counter per layer of a step follows the header
constexpr int kMaxLayers = 4096;
constexpr int kHeaderWords = kHdrPoolCounters + kMaxLayers;

// Layout of the global step axis of the decode step.  The first n_main steps are cut into W
// equal ranges of Q steps, one per wave.  The rest (one eighth, when every wave has enough
// work) is a pool of short ranges of P steps that waves take from a shared counter as they
// finish their own range: the waves of some parts of the chip stream measurably slower than
// others, and the pool lets the fast ones take up the slack.  U <= W static ranges hold steps
// (Q is rounded up); range r < U is static range r, range U + j is pool range j; partial
// records of range r and segment sigma go to slot r + sigma.
constexpr int kPoolRangeSteps = 16;
constexpr int kPoolShare = 8;
constexpr int kPoolMinStepsPerWave = 96;

struct StepLayout {
  int64_t N, n_main;
  int32_t Q, W, U, P, R;
};

__host__ __device__ inline StepLayout layout_of(int64_t N, int W, bool pool) {
  StepLayout l;
  l.N = N;
  l.W = W;
  l.P = kPoolRangeSteps;
  int64_t pool_steps = 0;
  if (pool && N >= (int64_t)kPoolMinStepsPerWave * W)
    pool_steps = N / kPoolShare / kPoolRangeSteps * kPoolRangeSteps;
  l.n_main = N - pool_steps;
  const int64_t q = (l.n_main + W - 1) / W;
  l.Q = (int32_t)(q > 1 ? q : 1);
  l.U = (int32_t)((l.n_main + l.Q - 1) / l.Q);
  l.R = (int32_t)(pool_steps / kPoolRangeSteps);
  return l;
}
// Step numbers fit 31 bits (the entry points refuse more steps), so the divisions are 32-bit.
__host__ __device__ inline int64_t range_of_step(const StepLayout& l, int64_t x) {
  const uint32_t u = (uint32_t)x, m = (uint32_t)l.n_main;
  return u < m ? u / (uint32_t)l.Q : l.U + (u - m) / (uint32_t)kPoolRangeSteps;
}
__host__ __device__ inline bool step_opens_range(const StepLayout& l, int64_t x) {
  const uint32_t u = (uint32_t)x, m = (uint32_t)l.n_main;
  return u < m ? u % (uint32_t)l.Q == 0 : (u - m) % (uint32_t)kPoolRangeSteps == 0;
}
__host__ __device__ inline bool step_closes_range(const StepLayout& l, int64_t x) {
  if (x == l.N - 1 || x == l.n_main - 1) return true;
  const uint32_t u = (uint32_t)x, m = (uint32_t)l.n_main;
  return u < m ? u % (uint32_t)l.Q == (uint32_t)l.Q - 1
               : (u - m) % (uint32_t)kPoolRangeSteps == (uint32_t)kPoolRangeSteps - 1;
}
// The layout as the plan kernel left it in the header.
__device__ inline StepLayout layout_from_header(const int32_t* header) {
  StepLayout l;
  l.N = header[kHdrSteps];
  l.n_main = header[kHdrMain];
  l.Q = header[kHdrPerWave];
  l.W = header[kHdrWaves];
  l.U = header[kHdrUsed];
  l.P = kPoolRangeSteps;
  l.R = header[kHdrPool];
  return l;
}
// Upper bound of the number of pool ranges when only a bound of the step count is known.
__host__ __device__ inline int64_t pool_ranges_bound(int64_t steps_bound) {
  return steps_bound / kPoolShare / kPoolRangeSteps + 1;
}

// Workspace map (byte offsets from the 256-byte aligned workspace base).
struct Workspace {
  size_t header;       // int32[kHeaderWords]: 64 header words, then one pool counter per layer
  size_t step_prefix;  // int32[S + 1]: exclusive scan of n_s
  size_t desc;         // int4[desc_capacity]
  size_t partial_ml;   // float2[slots * G]: (running max in log2 units, sum)
  size_t partial_acc;  // float[slots * G * D]
  size_t total;
};

// Workspace map of the multi-token (prefill / chunk) step.
struct PrefillWorkspace {
  size_t header, ranges, pt, ps, tile_first, tile_steps, tile_info, split_list,
      partial_ml, partial_acc, desc, total;
};

// Everything a kernel needs besides its buffers.
struct Params {
  int32_t S, Hq, Hkv, G, D, P, max_nb;
  float scale_log2;  // scale * log2(e): scores are kept in log2 units
  // The layout of the step axis when the host knows the lengths (n_steps >= 0); else n_steps is
  // -1 and the kernels read the layout the plan kernel left in the header.  The hint saves
  // every wave a dependent round trip to memory before its first descriptor load.
  int32_t n_steps;
  StepLayout lay;
  int32_t waves;  // W: static ranges of the step axis
  // this launch's pool counter (zero when the launch starts), or null: equal ranges only
  int32_t* pool_counter;
  // When > 0: wave w owns steps [r[w], r[w+1]) with r = header + ranges_off (int32 words), a
  // table the plan wrote, instead of the equal ranges [w*Q, (w+1)*Q)
  int32_t ranges_off;
  // Measurement aid: when not null, wave w stores the chip's constant-rate clock at its start
  // and end in wave_clock[2w], wave_clock[2w+1]
  unsigned long long* wave_clock;
  // Multi-token step: where runs that are whole segments write their finished rows
  // ([rows][Hq][D] fp32 and, if not null, [rows][Hq] log-sum-exp)
  float* out;
  float* lse;
  // Mixed batches of the multi-token step: streams that bring exactly one token go through the
  // decode kernels, the others through the multi-token kernels.  q_rows (decode side; null in
  // the plain decode step): stream s's query row and output row is q_rows[s] of the packed row
  // arrays instead of s.  skip_single (multi-token plan): such streams get no tiles.
  const int32_t* q_rows;
  int32_t skip_single;
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// K pool [P][Hkv][D/32][B][32], V pool [P][Hkv][B/4][D][4]; element offsets of granule (blk, h).
__host__ __device__ inline size_t granule_offset(int64_t blk, int h, int Hkv, int D) {
  return ((size_t)blk * Hkv + h) * (size_t)(kBlock * D);
}
__host__ __device__ inline int k_elem(int t, int d) {
  return ((d >> 5) * kBlock + t) * 32 + (d & 31);
}
__host__ __device__ inline int v_elem(int t, int d, int D) { return ((t >> 2) * D + d) * 4 + (t & 3); }

// The buffers of one layer's append, passed by value to the kernels that carry an append role.
// Plain mode (qkv == nullptr): k_new / v_new rows are copied.  Fused mode: the rows come from
// the packed [S][Hq + 2*Hkv][D] output of the QKV projection; q and k heads are rotated with
// the cos / sin rows of position L_s - 1, q goes to q_out, k and v into the cache.
struct AppendArgs {
  const uint16_t* k_new;
  const uint16_t* v_new;
  uint16_t* k_pool;
  uint16_t* v_pool;
  const uint16_t* qkv;
  const float* rope_cos;
  const float* rope_sin;
  uint16_t* q_out;
};

// Launchers implemented in the kernel translation units; each returns hipGetLastError().
hipError_t launch_append(const Params& p, const AppendArgs& a, const int32_t* bt,
                         const int32_t* lens, hipStream_t st);
hipError_t launch_plan_append(const Params& p, const int32_t* bt, const int32_t* lens, int waves,
                              int64_t desc_capacity, int64_t max_steps, int32_t* header,
                              int32_t* step_prefix, int4* desc, const AppendArgs& a,
                              hipStream_t st);
hipError_t launch_merge_append(const Params& p, const int32_t* header, const int32_t* step_prefix,
                               const float2* partial_ml, const float* partial_acc, float* out,
                               const int32_t* bt, const int32_t* lens, const AppendArgs& a,
                               hipStream_t st);
hipError_t launch_kv_gather(const Params& p, const void* k_pool, const void* v_pool,
                            const int32_t* bt, const int32_t* lens, const int64_t* row_offsets,
                            void* k_out, void* v_out, hipStream_t st);
hipError_t launch_plan(const Params& p, const int32_t* bt, const int32_t* lens, int waves,
                       int64_t desc_capacity, int64_t max_steps, int32_t* header,
                       int32_t* step_prefix, int4* desc, hipStream_t st);
PrefillWorkspace map_prefill_workspace(const Params& p, int ncg, int64_t tiles, int64_t slots,
                                       int64_t desc_capacity, int waves);
int prefill_column_groups(const Params& p, int max_new_tokens);
hipError_t launch_read_probe(const void* buf, size_t bytes, void* sink, hipStream_t st);
size_t prefill_desc_bytes();
hipError_t launch_kv_append_multi(const Params& p, int total_q, const void* k_new,
                                  const void* v_new, void* k_pool, void* v_pool,
                                  const int32_t* bt, const int32_t* lens, const int32_t* qo,
                                  hipStream_t st);
// launch_prefill does the plan kernels, the attention and merge kernels, or both
constexpr int kPrefillPlan = 1, kPrefillRun = 2;
// tile_streams: streams that have tiles (0: all); lens_single: where the plan leaves the masked
// lengths of a mixed batch (or null); max_tile_steps: most steps of any tile, all kv heads
hipError_t launch_prefill(const Params& p, const PrefillWorkspace& m, char* ws, int ncg,
                          int64_t tiles, int64_t steps, int64_t desc_capacity, int waves,
                          const void* q, const void* k_pool, const void* v_pool,
                          const int32_t* bt, const int32_t* lens, const int32_t* qo, float* out,
                          float* lse, hipStream_t st, hipEvent_t ev_before,
                          hipEvent_t ev_after, int phases, int64_t tile_streams,
                          int32_t* lens_single, int64_t max_tile_steps);
hipError_t launch_decode_mfma(const Params& p, int waves, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* header, const int4* desc,
                              float2* partial_ml, float* partial_acc, hipStream_t st);
hipError_t launch_decode_valu(const Params& p, int waves, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* header, const int4* desc,
                              float2* partial_ml, float* partial_acc, hipStream_t st);
hipError_t launch_merge(const Params& p, const int32_t* header, const int32_t* step_prefix,
                        const float2* partial_ml, const float* partial_acc, float* out,
                        float* lse, hipStream_t st);

}  // namespace vox
