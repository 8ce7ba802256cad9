// C-ABI entry points: host-side validation, split-K planning policy and launches.
// Nothing here allocates, synchronises or copies; every call only enqueues kernels.
#include <math.h>

#include "vox_common.hpp"

namespace vox {
namespace {

constexpr int kComputeUnits = 256;
constexpr int kWaveSlotsPerCu = 8;  // the decode kernels run two waves per SIMD
constexpr int kRoundsTarget = 6;    // aim for this many wave-items per resident wave slot

int validate(const vox_shape_t* s) {
  if (!s) return VOX_ERR_NULL;
  if (s->num_streams <= 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->num_blocks <= 0 ||
      s->max_blocks_per_stream <= 0)
    return VOX_ERR_SHAPE;
  if (s->num_q_heads % s->num_kv_heads != 0) return VOX_ERR_SHAPE;
  const int g = s->num_q_heads / s->num_kv_heads;
  if (g > 8) return VOX_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return VOX_ERR_SHAPE;
  if (s->block_size != kBlock) return VOX_ERR_SHAPE;
  if (!(s->scale == s->scale) || isinf(s->scale)) return VOX_ERR_ARG;
  if (s->decode_path < VOX_PATH_AUTO || s->decode_path > VOX_PATH_VALU) return VOX_ERR_ARG;
  if (s->chunk_blocks != 0 &&
      (s->chunk_blocks < 2 || (s->chunk_blocks & 1) || s->chunk_blocks > kMaxChunkBlocks))
    return VOX_ERR_ARG;
  return VOX_OK;
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
  return p;
}

int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Chunk length the library prefers for `total_blocks` blocks of context: enough wave-items
// to give every resident wave slot several of them, within [2, kMaxChunkBlocks], even.
int preferred_chunk(const vox_shape_t* s, int64_t total_blocks) {
  if (s->chunk_blocks) return s->chunk_blocks;
  const int64_t slots = (int64_t)kComputeUnits * kWaveSlotsPerCu * kRoundsTarget;
  int64_t ch = (total_blocks * s->num_kv_heads + slots - 1) / slots;
  ch = (ch + 1) & ~(int64_t)1;
  if (ch < 4) ch = 4;
  if (ch > kMaxChunkBlocks) ch = kMaxChunkBlocks;
  return (int)ch;
}

int64_t blocks_upper_bound(const vox_shape_t* s) {
  return (int64_t)s->num_streams * s->max_blocks_per_stream;
}

// Items the plan can produce when nothing but the shape is known.
int64_t items_bound(const vox_shape_t* s, int ch) {
  return (int64_t)s->num_streams * ceil_div(s->max_blocks_per_stream, ch);
}

int64_t items_exact(const vox_shape_t* s, const int32_t* lens_host, int ch) {
  int64_t n = 0;
  for (int i = 0; i < s->num_streams; ++i) {
    const int nb = ceil_div(lens_host[i] > 0 ? lens_host[i] : 0, kBlock);
    n += ceil_div(nb, ch);
  }
  return n;
}

Workspace map_workspace(const vox_shape_t* s, int64_t capacity) {
  Workspace w;
  size_t off = 0;
  w.header = off;
  off = align_up(off + 64 * sizeof(int32_t), 256);
  w.first_item = off;
  off = align_up(off + ((size_t)s->num_streams + 1) * sizeof(int32_t), 256);
  w.items = off;
  off = align_up(off + (size_t)capacity * sizeof(Item), 256);
  w.partial_ml = off;
  off = align_up(off + (size_t)capacity * s->num_q_heads * sizeof(float2), 256);
  w.partial_acc = off;
  off = align_up(off + (size_t)capacity * s->num_q_heads * s->head_dim * sizeof(float), 256);
  w.total = off;
  w.capacity = (int32_t)capacity;
  return w;
}

// Largest capacity whose map fits in `bytes` (0 if not even one item per stream fits).
int64_t capacity_for(const vox_shape_t* s, size_t bytes) {
  const size_t per_item = sizeof(Item) + (size_t)s->num_q_heads * (sizeof(float2) +
                                                                  s->head_dim * sizeof(float));
  const size_t fixed = map_workspace(s, 0).total + 3 * 256;
  if (bytes <= fixed) return 0;
  int64_t cap = (int64_t)((bytes - fixed) / per_item);
  while (cap > 0 && map_workspace(s, cap).total > bytes) --cap;
  if (cap > INT32_MAX / 64) cap = INT32_MAX / 64;
  return cap;
}

struct Plan {
  int chunk_blocks;
  int64_t max_items;  // upper bound of the number of items (exact with host lengths)
  Workspace ws;
};

int make_plan(const vox_shape_t* s, const int32_t* lens_host, size_t workspace_bytes, Plan* out) {
  const int64_t cap = capacity_for(s, workspace_bytes);
  int64_t total_blocks = 0;
  if (lens_host) {
    for (int i = 0; i < s->num_streams; ++i) {
      if (lens_host[i] < 0 || lens_host[i] > (int64_t)s->max_blocks_per_stream * kBlock)
        return VOX_ERR_ARG;
      total_blocks += ceil_div(lens_host[i], kBlock);
    }
  } else {
    total_blocks = blocks_upper_bound(s);
    if (total_blocks > s->num_blocks) total_blocks = s->num_blocks;
  }
  int ch = preferred_chunk(s, total_blocks);
  for (;;) {
    const int64_t n = lens_host ? items_exact(s, lens_host, ch) : items_bound(s, ch);
    if (n <= cap) {
      out->chunk_blocks = ch;
      out->max_items = n;
      out->ws = map_workspace(s, cap < INT32_MAX ? cap : INT32_MAX);
      return VOX_OK;
    }
    if (ch >= kMaxChunkBlocks || s->chunk_blocks) return VOX_ERR_WORKSPACE;
    ch += 2;
  }
}

int enqueue_decode(const vox_shape_t* s, const Params& p, const Plan& plan, char* ws,
                   const void* q, const void* k_pool, const void* v_pool, const int32_t* bt,
                   const int32_t* lens, float* out, float* lse, hipStream_t st,
                   hipEvent_t ev_before = nullptr, hipEvent_t ev_after = nullptr) {
  const int32_t* header = (const int32_t*)(ws + plan.ws.header);
  const int32_t* first_item = (const int32_t*)(ws + plan.ws.first_item);
  const Item* items = (const Item*)(ws + plan.ws.items);
  float2* pml = (float2*)(ws + plan.ws.partial_ml);
  float* pacc = (float*)(ws + plan.ws.partial_acc);
  const int64_t wave_items = plan.max_items * p.Hkv;
  if (ev_before && hipEventRecord(ev_before, st) != hipSuccess) return VOX_ERR_HIP;
  if (wave_items > 0) {
    hipError_t e = (s->decode_path == VOX_PATH_VALU)
                       ? launch_decode_valu(p, (int)wave_items, q, k_pool, v_pool, bt, lens,
                                            header, items, pml, pacc, st)
                       : launch_decode_mfma(p, (int)wave_items, q, k_pool, v_pool, bt, lens,
                                            header, items, pml, pacc, st);
    if (e != hipSuccess) return VOX_ERR_HIP;
  }
  if (ev_after && hipEventRecord(ev_after, st) != hipSuccess) return VOX_ERR_HIP;
  if (launch_merge(p, first_item, pml, pacc, out, lse, st) != hipSuccess) return VOX_ERR_HIP;
  return VOX_OK;
}

int enqueue_plan(const Params& p, const Plan& plan, char* ws, const int32_t* lens,
                 hipStream_t st) {
  hipError_t e = launch_plan(p, lens, plan.chunk_blocks, plan.ws.capacity,
                             (int32_t*)(ws + plan.ws.header), (int32_t*)(ws + plan.ws.first_item),
                             (Item*)(ws + plan.ws.items), st);
  return e == hipSuccess ? VOX_OK : VOX_ERR_HIP;
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
  const Params p = make_params(shape);
  return launch_kv_append(p, k_new, v_new, k_pool, v_pool, block_tables, context_lens,
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
  const Params p = make_params(shape);
  return launch_kv_gather(p, k_pool, v_pool, block_tables, context_lens, row_offsets, k_out,
                          v_out, (hipStream_t)hip_stream) == hipSuccess
             ? VOX_OK
             : VOX_ERR_HIP;
}

size_t vox_paged_decode_workspace_bytes(const vox_shape_t* shape) {
  if (validate(shape) != VOX_OK) return 0;
  int64_t nb = blocks_upper_bound(shape);
  if (nb > shape->num_blocks) nb = shape->num_blocks;
  const int ch = preferred_chunk(shape, nb);
  return map_workspace(shape, items_bound(shape, ch)).total + 4 * 256;
}

size_t vox_paged_decode_min_workspace_bytes(const vox_shape_t* shape) {
  if (validate(shape) != VOX_OK) return 0;
  const int ch = shape->chunk_blocks ? shape->chunk_blocks : kMaxChunkBlocks;
  return map_workspace(shape, items_bound(shape, ch)).total + 4 * 256;
}

int vox_paged_decode(const vox_shape_t* shape, const void* q, const void* k_pool,
                     const void* v_pool, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* context_lens_host, float* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return vox_paged_decode_profiled(shape, q, k_pool, v_pool, block_tables, context_lens,
                                   context_lens_host, out, lse, workspace, workspace_bytes,
                                   hip_stream, nullptr, nullptr);
}

int vox_paged_decode_profiled(const vox_shape_t* shape, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* block_tables,
                              const int32_t* context_lens, const int32_t* context_lens_host,
                              float* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream, void* event_before, void* event_after) {
  if (int rc = validate(shape)) return rc;
  if (!q || !k_pool || !v_pool || !block_tables || !context_lens || !out || !workspace)
    return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256) return VOX_ERR_ARG;
  Plan plan;
  if (int rc = make_plan(shape, context_lens_host, workspace_bytes, &plan)) return rc;
  const Params p = make_params(shape);
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  if (int rc = enqueue_plan(p, plan, ws, context_lens, st)) return rc;
  return enqueue_decode(shape, p, plan, ws, q, k_pool, v_pool, block_tables, context_lens, out,
                        lse, st, (hipEvent_t)event_before, (hipEvent_t)event_after);
}

int vox_decode_step(const vox_shape_t* shape, int32_t num_layers, const void* const* q,
                    const void* const* k_new, const void* const* v_new, void* const* k_pool,
                    void* const* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                    const int32_t* context_lens_host, float* const* out, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (int rc = validate(shape)) return rc;
  if (num_layers <= 0) return VOX_ERR_ARG;
  if (!q || !k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens || !out ||
      !workspace)
    return VOX_ERR_NULL;
  for (int l = 0; l < num_layers; ++l)
    if (!q[l] || !k_new[l] || !v_new[l] || !k_pool[l] || !v_pool[l] || !out[l])
      return VOX_ERR_NULL;
  if ((uintptr_t)workspace % 256) return VOX_ERR_ARG;
  Plan plan;
  if (int rc = make_plan(shape, context_lens_host, workspace_bytes, &plan)) return rc;
  const Params p = make_params(shape);
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  if (int rc = enqueue_plan(p, plan, ws, context_lens, st)) return rc;
  for (int l = 0; l < num_layers; ++l) {
    if (launch_kv_append(p, k_new[l], v_new[l], k_pool[l], v_pool[l], block_tables, context_lens,
                         st) != hipSuccess)
      return VOX_ERR_HIP;
    if (int rc = enqueue_decode(shape, p, plan, ws, q[l], k_pool[l], v_pool[l], block_tables,
                                context_lens, out[l], nullptr, st))
      return rc;
  }
  return VOX_OK;
}

const char* vox_strerror(int code) {
  switch (code) {
    case VOX_OK: return "ok";
    case VOX_ERR_NULL: return "a required pointer is NULL";
    case VOX_ERR_SHAPE: return "unsupported shape (need Hq % Hkv == 0, Hq/Hkv <= 8, head_dim 64 or 128, block_size 16, positive sizes)";
    case VOX_ERR_WORKSPACE: return "workspace too small (see vox_paged_decode_min_workspace_bytes)";
    case VOX_ERR_HIP: return "a HIP launch failed (see hipGetLastError)";
    case VOX_ERR_ARG: return "a scalar argument is out of range";
    default: return "unknown vox error code";
  }
}

}  // extern "C"
