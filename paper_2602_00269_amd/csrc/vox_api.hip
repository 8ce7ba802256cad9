// C-ABI entry points: host-side validation, split-K sizing and launches.
// Nothing here allocates device memory, synchronises or copies; every call only enqueues
// kernels.
#include <math.h>

#include <mutex>

#include "vox_common.hpp"

// Built-in scratch memory of vox_paged_decode_static: every GPU the library runs on holds its
// own copy of this array, at its own address, until the process ends.  In host code the name is
// only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[VOX_STATIC_SCRATCH_BYTES];

namespace vox {
namespace {

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
int static_scratch(void** out) {
  static std::mutex mu;
  static void* ptrs[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VOX_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return VOX_ERR_HIP;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return VOX_OK;
}

constexpr int kMaxSplitWaves = 1 << 20;

int validate(const vox_shape_t* s) {
  if (!s) return VOX_ERR_NULL;
  if (s->num_streams <= 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->num_blocks <= 0 ||
      s->max_blocks_per_stream <= 0)
    return VOX_ERR_SHAPE;
  if (s->num_streams > kMaxStreams) return VOX_ERR_SHAPE;
  if (s->num_q_heads % s->num_kv_heads != 0) return VOX_ERR_SHAPE;
  const int g = s->num_q_heads / s->num_kv_heads;
  if (g > 8) return VOX_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return VOX_ERR_SHAPE;
  if (s->block_size != kBlock) return VOX_ERR_SHAPE;
  if ((int64_t)s->num_blocks * s->num_kv_heads > INT32_MAX) return VOX_ERR_SHAPE;
  if ((int64_t)s->num_streams * s->num_kv_heads > INT32_MAX / 2) return VOX_ERR_SHAPE;
  if (!(s->scale == s->scale) || isinf(s->scale)) return VOX_ERR_ARG;
  if (s->decode_path < VOX_PATH_AUTO || s->decode_path > VOX_PATH_VALU) return VOX_ERR_ARG;
  if (s->split_waves < 0 || s->split_waves > kMaxSplitWaves) return VOX_ERR_ARG;
  return VOX_OK;
}

// Rows, pools and outputs are accessed with 16-byte vector loads and stores.
bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
template <class... T>
bool all_aligned16(const T*... ptrs) {
  return (aligned16(ptrs) && ...);
}

// Number of waves the step axis is dealt to: by default one per wave the decode kernel keeps
// resident on the whole chip, so the launch is a single balanced round.
int split_waves(const vox_shape_t* s) {
  int w = s->split_waves ? s->split_waves : kDesignWaveSlots;
  return (w + kWavesPerGroup - 1) / kWavesPerGroup * kWavesPerGroup;
}

Params make_params(const vox_shape_t* s) {
  Params p;
  p.S = s->num_streams;
  p.Hq = s->num_q_heads;
  p.Hkv = s->num_kv_heads;
  p.G = p.Hq / p.Hkv;
  p.D = s->head_dim;
  p.P = s->num_blocks;
  p.max_nb = s->max_blocks_per_stream;
  p.scale_log2 = s->scale * 1.44269504088896340736f;
  // A scale of zero (all scores equal) is replaced by one so small that every product with a
  // dot product still vanishes next to 1 in the exponent: the kernels may then rely on
  // scale * (+-inf) being an infinity, never NaN.
  if (p.scale_log2 == 0.f) p.scale_log2 = 0x1p-100f;
  p.n_steps = -1;
  p.lay = layout_of(0, 1, false);
  p.waves = split_waves(s);
  p.pool_counter = nullptr;
  p.ranges_off = 0;
  p.wave_clock = nullptr;
  p.out = nullptr;
  p.lse = nullptr;
  p.q_rows = nullptr;
  p.skip_single = 0;
  return p;
}

// Upper bound of the number of global steps when only the shape is known.
int64_t steps_bound(const vox_shape_t* s) {
  return (int64_t)s->num_streams * ((s->max_blocks_per_stream + 1) / 2) * s->num_kv_heads;
}

Workspace map_workspace(const vox_shape_t* s, int64_t desc_capacity) {
  const int g = s->num_q_heads / s->num_kv_heads;
  const size_t slots = (size_t)split_waves(s) + (size_t)pool_ranges_bound(steps_bound(s)) +
                       (size_t)s->num_streams * s->num_kv_heads;
  Workspace w;
  size_t off = 0;
  w.header = off;
  off = align_up(off + kHeaderWords * sizeof(int32_t), 256);
  w.step_prefix = off;
  off = align_up(off + ((size_t)s->num_streams + 1) * sizeof(int32_t), 256);
  w.partial_ml = off;
  off = align_up(off + slots * g * sizeof(float2), 256);
  w.partial_acc = off;
  off = align_up(off + slots * g * s->head_dim * sizeof(float), 256);
  w.desc = off;  // last, so that whatever the caller gives beyond the fixed part holds steps
  off = align_up(off + (size_t)desc_capacity * sizeof(int4), 256);
  w.total = off;
  return w;
}

// A captured call is replayed later, when the device lengths may have moved on (every decode
// step adds a token, and crossing a 32-token boundary changes the step count): nothing of the
// recorded launches may then depend on the host copy of the lengths.  While the stream is being
// captured the host copy is therefore ignored and the call behaves as if it were NULL: the
// kernels read the layout of the step axis from the plan's header, grids cover the shape's bound.
const int32_t* lens_for_planning(const int32_t* lens_host, hipStream_t st) {
  if (!lens_host) return nullptr;
  hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &status) != hipSuccess) {
    (void)hipGetLastError();  // e.g. the legacy default stream while another stream captures
    return nullptr;
  }
  return status == hipStreamCaptureStatusNone ? lens_host : nullptr;
}

struct Plan {
  int waves;
  int64_t desc_capacity;  // descriptors the workspace has room for
  int64_t max_steps;      // steps the plan kernel must be able to expand
  bool exact;             // max_steps is the exact step count (host lengths were given)
  Workspace ws;
};

// single_of: when not null (mixed batches), the host copy of q_offsets; only the streams that
// bring exactly one token count, the others are planned as empty.
int make_plan(const vox_shape_t* s, const int32_t* lens_host, size_t workspace_bytes, Plan* out,
              const int32_t* single_of = nullptr) {
  const size_t fixed = map_workspace(s, 0).total;
  if (workspace_bytes < fixed + sizeof(int4)) return VOX_ERR_WORKSPACE;
  const int64_t cap = (int64_t)((workspace_bytes - fixed) / sizeof(int4));
  int64_t need = steps_bound(s);
  if (lens_host) {
    need = 0;
    for (int i = 0; i < s->num_streams; ++i) {
      if (lens_host[i] < 0 || lens_host[i] > (int64_t)s->max_blocks_per_stream * kBlock)
        return VOX_ERR_ARG;
      if (single_of && single_of[i + 1] - single_of[i] != 1) continue;
      need += ((lens_host[i] + kBlock - 1) / kBlock + 1) / 2;
    }
    need *= s->num_kv_heads;
  }
  if (need > INT32_MAX) return VOX_ERR_SHAPE;
  if (need > cap) return VOX_ERR_WORKSPACE;
  out->waves = split_waves(s);
  out->desc_capacity = cap < INT32_MAX ? cap : INT32_MAX;
  out->max_steps = need;
  out->exact = lens_host != nullptr;
  out->ws = map_workspace(s, 0);
  return VOX_OK;
}

// With exact host-side knowledge of the step count, the layout of the step axis travels as a
// kernel argument (the plan kernel derives the same layout from the device lengths).
void set_step_hints(Params* p, const Plan& plan) {
  if (!plan.exact) return;
  p->n_steps = (int32_t)plan.max_steps;
  p->lay = layout_of(plan.max_steps, plan.waves, p->pool_counter != nullptr);
}

// The pool counter of layer l of a step (zeroed by the plan kernel).
int32_t* pool_counter(const Plan& plan, char* ws, int layer) {
  return (int32_t*)(ws + plan.ws.header) + kHdrPoolCounters + layer;
}

int enqueue_plan(const Params& p, const Plan& plan, char* ws, const int32_t* bt,
                 const int32_t* lens, hipStream_t st) {
  hipError_t e = launch_plan(p, bt, lens, plan.waves, plan.desc_capacity, plan.max_steps,
                             (int32_t*)(ws + plan.ws.header),
                             (int32_t*)(ws + plan.ws.step_prefix), (int4*)(ws + plan.ws.desc), st);
  return e == hipSuccess ? VOX_OK : VOX_ERR_HIP;
}

struct WsPtrs {
  int32_t* header;
  int32_t* step_prefix;
  int4* desc;
  float2* pml;
  float* pacc;
};

WsPtrs ws_ptrs(const Plan& plan, char* ws) {
  return WsPtrs{(int32_t*)(ws + plan.ws.header), (int32_t*)(ws + plan.ws.step_prefix),
                (int4*)(ws + plan.ws.desc), (float2*)(ws + plan.ws.partial_ml),
                (float*)(ws + plan.ws.partial_acc)};
}

// Append roles: rows that arrive as separate K and V tensors ...
AppendArgs plain_append(const void* k_new, const void* v_new, void* k_pool, void* v_pool) {
  return AppendArgs{(const uint16_t*)k_new, (const uint16_t*)v_new, (uint16_t*)k_pool,
                    (uint16_t*)v_pool, nullptr, nullptr, nullptr, nullptr};
}
// ... or as fused q|k|v rows that are rotated and split on the way (q goes to q_out).
AppendArgs rope_append(const void* qkv, const float* rope_cos, const float* rope_sin, void* q_out,
                       void* k_pool, void* v_pool) {
  return AppendArgs{nullptr, nullptr, (uint16_t*)k_pool, (uint16_t*)v_pool, (const uint16_t*)qkv,
                    rope_cos, rope_sin, (uint16_t*)q_out};
}
// The cos / sin tables must cover every position the shape admits: the kernels index them with
// L_s - 1 from device memory and cannot report a short table.
bool rope_table_ok(const vox_shape_t* s, int32_t rope_positions) {
  return rope_positions >= s->max_blocks_per_stream * kBlock;
}

// The split-K attention launch alone (the merge follows separately).
int enqueue_attention(const vox_shape_t* s, const Params& p, const Plan& plan, const WsPtrs& w,
                      const void* q, const void* k_pool, const void* v_pool, hipStream_t st,
                      hipEvent_t ev_before = nullptr, hipEvent_t ev_after = nullptr) {
  // no more waves than steps can exist (each launched wave without a range exits at once)
  int waves = plan.waves;
  if (plan.max_steps < waves)
    waves = (int)((plan.max_steps + kWavesPerGroup - 1) / kWavesPerGroup * kWavesPerGroup);
  if (ev_before && hipEventRecord(ev_before, st) != hipSuccess) return VOX_ERR_HIP;
  if (waves > 0) {
    hipError_t e = (s->decode_path == VOX_PATH_VALU)
                       ? launch_decode_valu(p, waves, q, k_pool, v_pool, w.header, w.desc, w.pml,
                                            w.pacc, st)
                       : launch_decode_mfma(p, waves, q, k_pool, v_pool, w.header, w.desc, w.pml,
                                            w.pacc, st);
    if (e != hipSuccess) return VOX_ERR_HIP;
  }
  if (ev_after && hipEventRecord(ev_after, st) != hipSuccess) return VOX_ERR_HIP;
  return VOX_OK;
}

// Mixed batches of the multi-token step.  A stream that brings exactly one token is a decode
// stream: the decode kernels (a pool of short ranges against the tail, three steps in flight,
// records kept in LDS) serve it better than a one-row tile of the multi-token kernel, so when
// there are enough of them they take those streams and the multi-token kernels the rest.  The
// workspace then holds, after the multi-token part: the masked lengths, the decode workspace.
// The split costs three more launches (about 15 us): measured against the single kernel it pays
// from about 32 k steps of single-token streams on (0.5 GB of K/V at head_dim 128).
constexpr int kMinSingleStreams = 32;
constexpr int64_t kMinSingleSteps = 32768;
size_t mixed_batch_base(size_t prefill_bytes, const vox_shape_t* s) {
  return align_up(prefill_bytes, 256) + align_up((size_t)s->num_streams * sizeof(int32_t), 256);
}

// The layers of a step.  q_of(l): layer l's query rows as the attention reads them;
// append_of(l): the append role of layer l.
// Launch chain: [plan + append(0)] attention(0) [merge(0) + append(1)] attention(1) ...
// merge(L-1).  Each bracket is one launch of two independent roles.
template <class QOf, class AppendOf>
int step_layers(const vox_shape_t* shape, int num_layers, QOf q_of, AppendOf append_of,
                void* const* k_pool, void* const* v_pool, const int32_t* block_tables,
                const int32_t* context_lens, const int32_t* context_lens_host, float* const* out,
                void* workspace, size_t workspace_bytes, hipStream_t st) {
  Plan plan;
  if (int rc = make_plan(shape, lens_for_planning(context_lens_host, st), workspace_bytes, &plan))
    return rc;
  Params p = make_params(shape);
  char* ws = (char*)workspace;
  p.pool_counter = pool_counter(plan, ws, 0);  // the plan zeroes every layer's counter
  set_step_hints(&p, plan);
  const WsPtrs w = ws_ptrs(plan, ws);
  if (launch_plan_append(p, block_tables, context_lens, plan.waves, plan.desc_capacity,
                         plan.max_steps, w.header, w.step_prefix, w.desc, append_of(0),
                         st) != hipSuccess)
    return VOX_ERR_HIP;
  for (int l = 0; l < num_layers; ++l) {
    p.pool_counter = pool_counter(plan, ws, l);
    if (int rc = enqueue_attention(shape, p, plan, w, q_of(l), k_pool[l], v_pool[l], st))
      return rc;
    hipError_t e = l + 1 < num_layers
                       ? launch_merge_append(p, w.header, w.step_prefix, w.pml, w.pacc, out[l],
                                             block_tables, context_lens, append_of(l + 1), st)
                       : launch_merge(p, w.header, w.step_prefix, w.pml, w.pacc, out[l], nullptr,
                                      st);
    if (e != hipSuccess) return VOX_ERR_HIP;
  }
  return VOX_OK;
}

// One decode call on a given workspace (the caller's, or the built-in scratch array).
int decode_call(const vox_shape_t* shape, const void* q, const void* k_pool, const void* v_pool,
                const int32_t* block_tables, const int32_t* context_lens,
                const int32_t* context_lens_host, float* out, float* lse, void* workspace,
                size_t workspace_bytes, void* hip_stream, void* event_before, void* event_after,
                uint64_t* wave_clock) {
  if (!q || !k_pool || !v_pool || !block_tables || !context_lens || !out || !workspace)
    return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256 || !all_aligned16(q, k_pool, v_pool, out)) return VOX_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  Plan plan;
  if (int rc = make_plan(shape, lens_for_planning(context_lens_host, st), workspace_bytes, &plan))
    return rc;
  Params p = make_params(shape);
  char* ws = (char*)workspace;
  p.pool_counter = pool_counter(plan, ws, 0);
  set_step_hints(&p, plan);
  p.wave_clock = (unsigned long long*)wave_clock;
  if (int rc = enqueue_plan(p, plan, ws, block_tables, context_lens, st)) return rc;
  const WsPtrs w = ws_ptrs(plan, ws);
  if (int rc = enqueue_attention(shape, p, plan, w, q, k_pool, v_pool, st,
                                 (hipEvent_t)event_before, (hipEvent_t)event_after))
    return rc;
  return launch_merge(p, w.header, w.step_prefix, w.pml, w.pacc, out, lse, st) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

// The multi-token step: its plan (phases & kPrefillPlan: everything that depends only on the
// lengths, the offsets and the block tables), its attention and merge on one layer's buffers
// (phases & kPrefillRun), or both.  `layer` selects the pool counter of the decode part of a
// mixed batch.
int prefill_call(const vox_shape_t* shape, int phases, int layer, const void* q,
                 const void* k_pool, const void* v_pool, const int32_t* block_tables,
                 const int32_t* context_lens, const int32_t* q_offsets,
                 const int32_t* context_lens_host, const int32_t* q_offsets_host, float* out,
                 float* lse, void* workspace, size_t workspace_bytes, void* hip_stream,
                 void* event_before, void* event_after) {
  if (int rc = validate(shape)) return rc;
  if (!context_lens_host || !q_offsets_host) return VOX_ERR_NULL;
  if (q_offsets_host[shape->num_streams] == 0 && q_offsets_host[0] == 0)
    return VOX_OK;  // no query rows: nothing to compute, the row arrays may be empty (NULL)
  const bool run = (phases & kPrefillRun) != 0;
  if (!block_tables || !context_lens || !q_offsets || !workspace) return VOX_ERR_NULL;
  if (run && (!q || !k_pool || !v_pool || !out)) return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256 || (run && !all_aligned16(q, k_pool, v_pool, out)))
    return VOX_ERR_ARG;
  Params p = make_params(shape);
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  // exact tile and step counts from the host copies (the scheduler that admits a prompt
  // knows its length)
  if (q_offsets_host[0] != 0) return VOX_ERR_ARG;
  int singles = 0;
  int64_t single_steps = 0;
  for (int s = 0; s < p.S; ++s) {
    const int64_t n = (int64_t)q_offsets_host[s + 1] - q_offsets_host[s];
    const int64_t L = context_lens_host[s];
    if (n < 0 || n > L || L > (int64_t)shape->max_blocks_per_stream * kBlock) return VOX_ERR_ARG;
    if (n == 1) {
      ++singles;
      single_steps += (L + kStepTokens - 1) / kStepTokens * p.Hkv;
    }
  }
  const bool split = singles >= kMinSingleStreams && single_steps >= kMinSingleSteps &&
                     shape->decode_path != VOX_PATH_VALU;
  const int waves = split_waves(shape);
  // Two passes at most: with the single-token streams left to the decode kernels when there are
  // enough of them and the workspace has room for both parts, else with every stream here.
  for (int mixed = split ? 1 : 0; mixed >= 0; --mixed) {
    int64_t max_new = 0, tile_streams = 0;
    for (int s = 0; s < p.S; ++s) {
      const int64_t n = (int64_t)q_offsets_host[s + 1] - q_offsets_host[s];
      if (mixed && n == 1) continue;
      if (n > max_new) max_new = n;
      tile_streams += n > 0;
    }
    const int ncg = prefill_column_groups(p, (int)(max_new < INT32_MAX ? max_new : INT32_MAX));
    const int tq = (16 / p.G) * ncg;
    int64_t tiles = 0, steps = 0, max_tile_steps = 1;
    for (int s = 0; s < p.S; ++s) {
      const int64_t n = (int64_t)q_offsets_host[s + 1] - q_offsets_host[s];
      if (mixed && n == 1) continue;
      const int64_t L = context_lens_host[s];
      const int64_t nt = (n + tq - 1) / tq;
      if (n > 0 && (L + kStepTokens - 1) / kStepTokens * p.Hkv > max_tile_steps)
        max_tile_steps = (L + kStepTokens - 1) / kStepTokens * p.Hkv;
      for (int64_t tau = 0; tau < nt; ++tau) {
        const int64_t ctx = L - n + (n < (tau + 1) * tq ? n : (tau + 1) * tq);
        steps += (ctx + kStepTokens - 1) / kStepTokens;
      }
      tiles += nt;
    }
    steps *= p.Hkv;
    if (steps > INT32_MAX || tiles * p.Hkv > INT32_MAX / 2) return VOX_ERR_SHAPE;
    const int64_t slots = waves + tiles * p.Hkv;
    const PrefillWorkspace m = map_prefill_workspace(p, ncg, tiles, slots, steps, waves);
    if (!mixed) {
      if (m.total > workspace_bytes) return VOX_ERR_WORKSPACE;
      return launch_prefill(p, m, ws, ncg, tiles, steps, steps, waves, q, k_pool, v_pool,
                            block_tables, context_lens, q_offsets, out, lse, st,
                            (hipEvent_t)event_before, (hipEvent_t)event_after, phases, 0,
                            nullptr, max_tile_steps) == hipSuccess
                 ? VOX_OK
                 : VOX_ERR_HIP;
    }
    // the decode part: masked lengths on both sides, its own workspace behind the multi-token one
    const size_t lens_off = align_up(m.total, 256), dec_off = mixed_batch_base(m.total, shape);
    if (dec_off >= workspace_bytes) continue;
    Plan plan;
    if (make_plan(shape, context_lens_host, workspace_bytes - dec_off, &plan, q_offsets_host) !=
        VOX_OK)
      continue;
    int32_t* lens_single = (int32_t*)(ws + lens_off);
    char* dws = ws + dec_off;
    Params pd = p;  // the decode kernels' view
    pd.q_rows = q_offsets;
    pd.pool_counter = pool_counter(plan, dws, layer);  // the plan zeroes every layer's counter
    set_step_hints(&pd, plan);
    p.skip_single = 1;  // the multi-token plan's view
    if (phases & kPrefillPlan) {
      // the multi-token plan's first kernel also writes the masked lengths
      if (launch_prefill(p, m, ws, ncg, tiles, steps, steps, waves, q, k_pool, v_pool,
                         block_tables, context_lens, q_offsets, out, lse, st, nullptr, nullptr,
                         kPrefillPlan, tile_streams, lens_single, max_tile_steps) != hipSuccess)
        return VOX_ERR_HIP;
      if (int rc = enqueue_plan(pd, plan, dws, block_tables, lens_single, st)) return rc;
    }
    if (!run) return VOX_OK;
    const WsPtrs w = ws_ptrs(plan, dws);
    // the events enclose both attention kernels
    hipEvent_t after_decode = tiles > 0 ? nullptr : (hipEvent_t)event_after;
    if (int rc = enqueue_attention(shape, pd, plan, w, q, k_pool, v_pool, st,
                                   (hipEvent_t)event_before, after_decode))
      return rc;
    if (launch_prefill(p, m, ws, ncg, tiles, steps, steps, waves, q, k_pool, v_pool, block_tables,
                       context_lens, q_offsets, out, lse, st, nullptr, (hipEvent_t)event_after,
                       kPrefillRun, tile_streams, nullptr, max_tile_steps) != hipSuccess)
      return VOX_ERR_HIP;
    return launch_merge(pd, w.header, w.step_prefix, w.pml, w.pacc, out, lse, st) == hipSuccess
               ? VOX_OK
               : VOX_ERR_HIP;
  }
  return VOX_ERR_WORKSPACE;  // not reached: the pass with every stream here returns
}

}  // namespace
}  // namespace vox

using namespace vox;

extern "C" {

int vox_kv_append(const vox_shape_t* shape, const void* k_new, const void* v_new, void* k_pool,
                  void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                  void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens)
    return VOX_ERR_NULL;
  if (!all_aligned16(k_new, v_new, k_pool, v_pool)) return VOX_ERR_ARG;
  const Params p = make_params(shape);
  return launch_append(p, plain_append(k_new, v_new, k_pool, v_pool), block_tables, context_lens,
                       (hipStream_t)hip_stream) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

int vox_kv_gather(const vox_shape_t* shape, const void* k_pool, const void* v_pool,
                  const int32_t* block_tables, const int32_t* context_lens,
                  const int64_t* row_offsets, void* k_out, void* v_out, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (!k_pool || !v_pool || !block_tables || !context_lens || !row_offsets || !k_out || !v_out)
    return VOX_ERR_NULL;
  if (!all_aligned16(k_pool, v_pool, k_out, v_out)) return VOX_ERR_ARG;
  const Params p = make_params(shape);
  return launch_kv_gather(p, k_pool, v_pool, block_tables, context_lens, row_offsets, k_out,
                          v_out, (hipStream_t)hip_stream) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

size_t vox_paged_decode_workspace_bytes(const vox_shape_t* shape) {
  if (validate(shape) != VOX_OK) return 0;
  return map_workspace(shape, steps_bound(shape)).total;
}

int vox_paged_decode(const vox_shape_t* shape, const void* q, const void* k_pool,
                     const void* v_pool, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* context_lens_host, float* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return vox_paged_decode_profiled(shape, q, k_pool, v_pool, block_tables, context_lens,
                                   context_lens_host, out, lse, workspace, workspace_bytes,
                                   hip_stream, nullptr, nullptr, nullptr);
}

int vox_paged_decode_profiled(const vox_shape_t* shape, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* block_tables,
                              const int32_t* context_lens, const int32_t* context_lens_host,
                              float* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream, void* event_before, void* event_after,
                              uint64_t* wave_clock) {
  if (int rc = validate(shape)) return rc;
  if (!workspace) return VOX_ERR_NULL;
  return decode_call(shape, q, k_pool, v_pool, block_tables, context_lens, context_lens_host, out,
                     lse, workspace, workspace_bytes, hip_stream, event_before, event_after,
                     wave_clock);
}

int vox_paged_decode_static(const vox_shape_t* shape, const void* q, const void* k_pool,
                            const void* v_pool, const int32_t* block_tables,
                            const int32_t* context_lens, const int32_t* context_lens_host,
                            float* out, float* lse, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (!q || !k_pool || !v_pool || !block_tables || !context_lens || !out) return VOX_ERR_NULL;
  void* ws = nullptr;
  if (int rc = static_scratch(&ws)) return rc;
  const int rc = decode_call(shape, q, k_pool, v_pool, block_tables, context_lens,
                             context_lens_host, out, lse, ws, VOX_STATIC_SCRATCH_BYTES,
                             hip_stream, nullptr, nullptr, nullptr);
  return rc == VOX_ERR_WORKSPACE ? VOX_ERR_SCRATCH : rc;
}


int vox_decode_step(const vox_shape_t* shape, int32_t num_layers, const void* const* q,
                    const void* const* k_new, const void* const* v_new, void* const* k_pool,
                    void* const* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                    const int32_t* context_lens_host, float* const* out, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (num_layers <= 0 || num_layers > kMaxLayers) return VOX_ERR_ARG;
  if (!q || !k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens || !out ||
      !workspace)
    return VOX_ERR_NULL;
  for (int l = 0; l < num_layers; ++l)
    if (!q[l] || !k_new[l] || !v_new[l] || !k_pool[l] || !v_pool[l] || !out[l])
      return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256) return VOX_ERR_ARG;
  for (int l = 0; l < num_layers; ++l)
    if (!all_aligned16(q[l], k_new[l], v_new[l], k_pool[l], v_pool[l], out[l])) return VOX_ERR_ARG;
  return step_layers(
      shape, num_layers, [&](int l) { return q[l]; },
      [&](int l) { return plain_append(k_new[l], v_new[l], k_pool[l], v_pool[l]); }, k_pool,
      v_pool, block_tables, context_lens, context_lens_host, out, workspace, workspace_bytes,
      (hipStream_t)hip_stream);
}

int vox_decode_plan(const vox_shape_t* shape, const int32_t* block_tables,
                    const int32_t* context_lens, const int32_t* context_lens_host, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (!block_tables || !context_lens || !workspace) return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256) return VOX_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  Plan plan;
  if (int rc = make_plan(shape, lens_for_planning(context_lens_host, st), workspace_bytes, &plan))
    return rc;
  Params p = make_params(shape);
  p.pool_counter = pool_counter(plan, (char*)workspace, 0);  // the plan zeroes every layer's counter
  return enqueue_plan(p, plan, (char*)workspace, block_tables, context_lens, st);
}

int vox_decode_layer(const vox_shape_t* shape, int32_t layer, const void* q, const void* k_new,
                     const void* v_new, void* k_pool, void* v_pool, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* context_lens_host, float* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (layer < 0 || layer >= kMaxLayers) return VOX_ERR_ARG;
  if (!q || !k_pool || !v_pool || !block_tables || !context_lens || !out || !workspace)
    return VOX_ERR_NULL;
  if ((k_new == nullptr) != (v_new == nullptr)) return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256 || !all_aligned16(q, k_pool, v_pool, out)) return VOX_ERR_ARG;
  if (k_new && !all_aligned16(k_new, v_new)) return VOX_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  Plan plan;
  if (int rc = make_plan(shape, lens_for_planning(context_lens_host, st), workspace_bytes, &plan))
    return rc;
  Params p = make_params(shape);
  char* ws = (char*)workspace;
  p.pool_counter = pool_counter(plan, ws, layer);
  set_step_hints(&p, plan);
  const WsPtrs w = ws_ptrs(plan, ws);
  if (k_new && launch_append(p, plain_append(k_new, v_new, k_pool, v_pool), block_tables,
                             context_lens, st) != hipSuccess)
    return VOX_ERR_HIP;
  if (int rc = enqueue_attention(shape, p, plan, w, q, k_pool, v_pool, st)) return rc;
  return launch_merge(p, w.header, w.step_prefix, w.pml, w.pacc, out, lse, st) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

int vox_read_probe(const void* buf, size_t bytes, void* sink, void* hip_stream) {
  if (!buf || !sink) return VOX_ERR_NULL;
  if (bytes == 0 || bytes % 16 || (uintptr_t)buf % 16) return VOX_ERR_ARG;
  return launch_read_probe(buf, bytes, sink, (hipStream_t)hip_stream) == hipSuccess ? VOX_OK
                                                                                   : VOX_ERR_HIP;
}

int vox_rope_append(const vox_shape_t* shape, const void* qkv, const float* rope_cos,
                    const float* rope_sin, int32_t rope_positions, void* q_out, void* k_pool,
                    void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                    void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (!qkv || !rope_cos || !rope_sin || !q_out || !k_pool || !v_pool || !block_tables ||
      !context_lens)
    return VOX_ERR_NULL;
  if (!rope_table_ok(shape, rope_positions)) return VOX_ERR_ARG;
  if (!all_aligned16(qkv, rope_cos, rope_sin, q_out, k_pool, v_pool)) return VOX_ERR_ARG;
  const Params p = make_params(shape);
  return launch_append(p, rope_append(qkv, rope_cos, rope_sin, q_out, k_pool, v_pool),
                       block_tables, context_lens, (hipStream_t)hip_stream) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

int vox_decode_step_rope(const vox_shape_t* shape, int32_t num_layers, const void* const* qkv,
                         const float* rope_cos, const float* rope_sin, int32_t rope_positions,
                         void* const* q_rot, void* const* k_pool, void* const* v_pool,
                         const int32_t* block_tables, const int32_t* context_lens,
                         const int32_t* context_lens_host, float* const* out, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (num_layers <= 0 || num_layers > kMaxLayers) return VOX_ERR_ARG;
  if (!qkv || !rope_cos || !rope_sin || !q_rot || !k_pool || !v_pool || !block_tables ||
      !context_lens || !out || !workspace)
    return VOX_ERR_NULL;
  for (int l = 0; l < num_layers; ++l)
    if (!qkv[l] || !q_rot[l] || !k_pool[l] || !v_pool[l] || !out[l]) return VOX_ERR_NULL;
  if (!rope_table_ok(shape, rope_positions)) return VOX_ERR_ARG;
  if ((uintptr_t)workspace % 256 || !all_aligned16(rope_cos, rope_sin)) return VOX_ERR_ARG;
  for (int l = 0; l < num_layers; ++l)
    if (!all_aligned16(qkv[l], q_rot[l], k_pool[l], v_pool[l], out[l])) return VOX_ERR_ARG;
  return step_layers(
      shape, num_layers, [&](int l) { return (const void*)q_rot[l]; },
      [&](int l) {
        return rope_append(qkv[l], rope_cos, rope_sin, q_rot[l], k_pool[l], v_pool[l]);
      },
      k_pool, v_pool, block_tables, context_lens, context_lens_host, out, workspace,
      workspace_bytes, (hipStream_t)hip_stream);
}

size_t vox_paged_prefill_workspace_bytes(const vox_shape_t* shape, int32_t total_q) {
  if (validate(shape) != VOX_OK || total_q < 0) return 0;
  const Params p = make_params(shape);
  const int64_t tiles = (int64_t)total_q + shape->num_streams;  // every tile holds >= 1 row
  const int64_t steps = tiles * ((shape->max_blocks_per_stream + 1) / 2) * shape->num_kv_heads;
  const int64_t slots = split_waves(shape) + tiles * shape->num_kv_heads;
  // the widest records any call with this many rows may use: a smaller largest chunk can pick a
  // wider tile than the largest possible one does
  int ncg = 1;
  const int tq = 16 / p.G;
  for (int want = 1; want <= 32 && (want - 1) * tq < total_q; ++want) {
    const int rows = want * tq < total_q ? want * tq : total_q;
    const int c = prefill_column_groups(p, rows);
    if (c > ncg) ncg = c;
  }
  // a mixed batch also runs the decode kernels on the streams that bring one token
  return mixed_batch_base(map_prefill_workspace(p, ncg, tiles, slots, steps, split_waves(shape)).total,
                          shape) +
         map_workspace(shape, steps_bound(shape)).total;
}

int vox_kv_append_multi(const vox_shape_t* shape, const void* k_new, const void* v_new,
                        void* k_pool, void* v_pool, const int32_t* block_tables,
                        const int32_t* context_lens, const int32_t* q_offsets, int32_t total_q,
                        void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (total_q < 0) return VOX_ERR_ARG;
  if (total_q == 0) return VOX_OK;  // no rows: the row arrays may be empty (NULL)
  if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens || !q_offsets)
    return VOX_ERR_NULL;
  if (!all_aligned16(k_new, v_new, k_pool, v_pool)) return VOX_ERR_ARG;
  const Params p = make_params(shape);
  return launch_kv_append_multi(p, total_q, k_new, v_new, k_pool, v_pool, block_tables,
                                context_lens, q_offsets, (hipStream_t)hip_stream) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

int vox_paged_prefill(const vox_shape_t* shape, const void* q, const void* k_pool,
                      const void* v_pool, const int32_t* block_tables,
                      const int32_t* context_lens, const int32_t* q_offsets,
                      const int32_t* context_lens_host, const int32_t* q_offsets_host,
                      float* out, float* lse, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  return vox_paged_prefill_profiled(shape, q, k_pool, v_pool, block_tables, context_lens,
                                    q_offsets, context_lens_host, q_offsets_host, out, lse,
                                    workspace, workspace_bytes, hip_stream, nullptr, nullptr);
}

int vox_paged_prefill_profiled(const vox_shape_t* shape, const void* q, const void* k_pool,
                               const void* v_pool, const int32_t* block_tables,
                               const int32_t* context_lens, const int32_t* q_offsets,
                               const int32_t* context_lens_host, const int32_t* q_offsets_host,
                               float* out, float* lse, void* workspace, size_t workspace_bytes,
                               void* hip_stream, void* event_before, void* event_after) {
  return prefill_call(shape, kPrefillPlan | kPrefillRun, 0, q, k_pool, v_pool, block_tables,
                      context_lens, q_offsets, context_lens_host, q_offsets_host, out, lse,
                      workspace, workspace_bytes, hip_stream, event_before, event_after);
}

int vox_prefill_plan(const vox_shape_t* shape, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* q_offsets,
                     const int32_t* context_lens_host, const int32_t* q_offsets_host,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  return prefill_call(shape, kPrefillPlan, 0, nullptr, nullptr, nullptr, block_tables,
                      context_lens, q_offsets, context_lens_host, q_offsets_host, nullptr, nullptr,
                      workspace, workspace_bytes, hip_stream, nullptr, nullptr);
}

int vox_prefill_layer(const vox_shape_t* shape, int32_t layer, const void* q, const void* k_new,
                      const void* v_new, void* k_pool, void* v_pool, const int32_t* block_tables,
                      const int32_t* context_lens, const int32_t* q_offsets,
                      const int32_t* context_lens_host, const int32_t* q_offsets_host, float* out,
                      float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (layer < 0 || layer >= kMaxLayers) return VOX_ERR_ARG;
  if (!q_offsets_host || (k_new == nullptr) != (v_new == nullptr)) return VOX_ERR_NULL;
  if (k_new) {
    const int64_t rows = (int64_t)q_offsets_host[shape->num_streams] - q_offsets_host[0];
    if (rows < 0 || rows > INT32_MAX) return VOX_ERR_ARG;
    if (int rc = vox_kv_append_multi(shape, k_new, v_new, k_pool, v_pool, block_tables,
                                     context_lens, q_offsets, (int32_t)rows, hip_stream))
      return rc;
  }
  return prefill_call(shape, kPrefillRun, layer, q, k_pool, v_pool, block_tables, context_lens,
                      q_offsets, context_lens_host, q_offsets_host, out, lse, workspace,
                      workspace_bytes, hip_stream, nullptr, nullptr);
}

const char* vox_strerror(int code) {
  switch (code) {
    case VOX_OK: return "ok";
    case VOX_ERR_NULL: return "a required pointer is NULL";
    case VOX_ERR_SHAPE: return "unsupported shape (need Hq % Hkv == 0, Hq/Hkv <= 8, head_dim 64 or 128, block_size 16, 0 < streams <= 8192, positive sizes)";
    case VOX_ERR_WORKSPACE: return "workspace too small (see vox_paged_decode_workspace_bytes)";
    case VOX_ERR_HIP: return "a HIP launch failed (see hipGetLastError)";
    case VOX_ERR_ARG: return "a scalar argument is out of range, or a tensor is not 16-byte aligned";
    case VOX_ERR_SCRATCH: return "the call needs more than the VOX_STATIC_SCRATCH_BYTES of built-in scratch memory: use the entry point that takes a caller workspace";
    default: return "unknown vox error code";
  }
}

}  // extern "C"
