// Shared declarations of the HIP library: kernel parameter block, workspace map and the
// cache-layout index helpers.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vox.h"

namespace vox {

constexpr int kBlock = 16;         // tokens per KV block
constexpr int kWave = 64;          // lanes per wavefront
constexpr int kWavesPerGroup = 4;  // decode / merge workgroups are 4 independent waves
constexpr int kMaxChunkBlocks = 64;  // a wave keeps its chunk's block ids in one VGPR
constexpr int kStepTokens = 32;      // tokens consumed per MFMA step (two blocks)

// One split-K work item: `nblocks` consecutive logical blocks of one stream.  Each item is
// processed once per kv head; wave-item id = item * Hkv + h.
struct Item {
  int32_t stream;
  int32_t first_block;
  int32_t nblocks;
  int32_t pad;
};

// Workspace map (byte offsets from the 256-byte aligned workspace base).
struct Workspace {
  size_t header;       // int32[64]: [0] number of items, [1] chunk_blocks, [2] overflow flag
  size_t first_item;   // int32[S + 1]: exclusive scan of per-stream item counts
  size_t items;        // Item[capacity]
  size_t partial_ml;   // float2[capacity * Hq]: (running max in log2 units, sum)
  size_t partial_acc;  // float[capacity * Hq * D]
  size_t total;
  int32_t capacity;    // items the map has room for
};

// Everything a kernel needs besides its buffers.
struct Params {
  int32_t S, Hq, Hkv, G, D, P, max_nb;
  float scale_log2;  // scale * log2(e): scores are kept in log2 units
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// K pool [P][Hkv][D/8][B][8], V pool [P][Hkv][D][B]; element offsets of granule (blk, h).
__host__ __device__ inline size_t granule_offset(int64_t blk, int h, int Hkv, int D) {
  return ((size_t)blk * Hkv + h) * (size_t)(kBlock * D);
}
__host__ __device__ inline int k_elem(int t, int d) { return ((d >> 3) * kBlock + t) * 8 + (d & 7); }
__host__ __device__ inline int v_elem(int t, int d) { return d * kBlock + t; }

// Launchers implemented in the kernel translation units; each returns hipGetLastError().
hipError_t launch_kv_append(const Params& p, const void* k_new, const void* v_new, void* k_pool,
                            void* v_pool, const int32_t* bt, const int32_t* lens,
                            hipStream_t st);
hipError_t launch_kv_gather(const Params& p, const void* k_pool, const void* v_pool,
                            const int32_t* bt, const int32_t* lens, const int64_t* row_offsets,
                            void* k_out, void* v_out, hipStream_t st);
hipError_t launch_plan(const Params& p, const int32_t* lens, int chunk_blocks, int capacity,
                       int32_t* header, int32_t* first_item, Item* items, hipStream_t st);
hipError_t launch_decode_mfma(const Params& p, int max_wave_items, const void* q,
                              const void* k_pool, const void* v_pool, const int32_t* bt,
                              const int32_t* lens, const int32_t* header, const Item* items,
                              float2* partial_ml, float* partial_acc, hipStream_t st);
hipError_t launch_decode_valu(const Params& p, int max_wave_items, const void* q,
                              const void* k_pool, const void* v_pool, const int32_t* bt,
                              const int32_t* lens, const int32_t* header, const Item* items,
                              float2* partial_ml, float* partial_acc, hipStream_t st);
hipError_t launch_merge(const Params& p, const int32_t* first_item, const float2* partial_ml,
                        const float* partial_acc, float* out, float* lse, hipStream_t st);

}  // namespace vox
