// The split-K decode kernel skeleton shared by the MFMA and VALU arithmetic.
//
// A wave owns the global steps [w*Q, (w+1)*Q) of the static part of the step axis (or a range
// from the plan's table), then takes short ranges from a shared pool until it is used up.  It
// walks a range as one flat software pipeline: the K/V loads of step i + NBUF are issued while
// step i is computed, across segment boundaries, so the load queue never drains inside a range.  Step descriptors are wave-uniform:
// they come in through scalar loads a few steps ahead and live in scalar registers.  When a run
// of a segment ends inside the range its partial record is stored and the accumulators are
// reset; the query rows of the next run are fetched one step ahead.
//
// `Math` supplies the registers and arithmetic of one step:
//   struct Q (query rows in flight), struct Regs (one step of K/V), struct State;
//   struct Desc (step descriptor) with static accessors ga/gb/meta/sigma; columns(params);
//   Math(lane, params); load_q(Q&, State&, q, desc): issued right after the last step of the
//   previous run was computed (the state's own query registers are dead by then, so a Math may
//   load straight into them and leave Q empty); install_q(State&, Q&) at the run's first step;
//   issue(Regs&, k_pool, v_pool, ga, gb); reset(State&); compute(State&, Regs&, desc);
//   used_columns(desc): leading record columns that carry query rows (the rest is not stored);
//   finish(State&, float* acc, float* ml): writes the run's [columns][D] accumulators to acc
//   and its [columns] (max, sum) pairs to ml (an LDS record, or global memory when a record
//   does not fit the LDS buffer); kDirect: a step may carry kMetaWhole (its run is the whole
//   segment), then finish_rows(State&, desc) writes the finished rows instead of a record.
//   kSelfMerge: the wave that stores the last record of a segment merges the segment's records
//   and writes its output rows (decode step; the multi-token step has its own merge kernel).
//   kFusedAppend: patch_new_token(Regs&, desc) replaces, in the registers of a stream's last
//   step, the newest token's K / V values by its rows of k_new / v_new; the skeleton writes
//   those rows into the pools when the wave has finished its ranges.
#pragma once

#include "vox_merge.hpp"

namespace vox {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// KV data is read exactly once per step: non-temporal loads keep it from displacing the
// descriptors, queries and partial records in the caches.
template <bool STREAM>
__device__ inline u32x4 kv_load(const uint16_t* p) {
  if (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return *reinterpret_cast<const u32x4*>(p);
}

// Wave-private LDS buffer of finished partial records.  A global store issued in the middle of
// the load pipeline sits in the same in-order vector-memory counter as the K/V loads, and its
// acknowledgement is slow while the chip streams at full rate: every later load would wait
// behind it.  Records are therefore kept in LDS ([G][D] accumulators then [G] (max, sum)
// pairs, the same shape as a global record) and copied out when the wave has finished its
// range, or earlier if the buffer fills up (then only when the next record needs the room, so
// the last records of a wave always leave after its last load: stores that reach HBM while the
// chip streams reads cost far more than their bytes).  `cols` is the number of (query row,
// head) columns a record holds.  Each Math states the floats per wave it wants
// (`Math::kStashFloats`; four waves share the 160 KB of a CU).

struct PartialStash {
  float* mem;    // this wave's LDS area
  int rec;       // floats per record: cols * (D + 2)
  int gd;        // cols * D
  int cap;       // records that fit
  int count;     // records held
  int slots;     // lane r holds the slot id of record r
  int used;      // ... and the number of leading columns of it that carry query rows
  int sigs;      // ... and its segment
  int lane;

  __device__ PartialStash(float* mem_, int floats, int cols, int D, int lane_)
      : mem(mem_), rec(cols * (D + 2)), gd(cols * D), cap(floats / (cols * (D + 2))),
        count(0), slots(0), used(0), sigs(0), lane(lane_) {}

  // LDS area of the record being added (older records are stored first if the buffer is
  // full); the caller fills [col][d] at col*D + d and the (max, sum) pair of column col at
  // gd + 2*col, then calls commit().
  __device__ float* next(float2* __restrict__ pml, float* __restrict__ pacc) {
    if (count == cap) flush(pml, pacc);
    return mem + count * rec;
  }
  __device__ bool full() const { return count == cap; }

  __device__ void commit(int slot, int used_cols, int sigma) {
    if (lane == count) {
      slots = slot;
      used = used_cols;
      sigs = sigma;
    }
    ++count;
  }

  __device__ void flush(float2* __restrict__ pml, float* __restrict__ pacc) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int r = 0; r < count; ++r) {
      const int slot = __builtin_amdgcn_readlane(slots, r);
      const int floats = __builtin_amdgcn_readlane(used, r) * (gd / ((rec - gd) / 2));
      const float* src = mem + r * rec;
      float* dst = pacc + (size_t)slot * gd;
      for (int x = lane * 4; x < floats; x += kWave * 4)
        *reinterpret_cast<float4*>(dst + x) = *reinterpret_cast<const float4*>(src + x);
      for (int x = lane; 2 * x < rec - gd; x += kWave)
        pml[(size_t)slot * (rec - gd) / 2 + x] =
            *reinterpret_cast<const float2*>(src + gd + 2 * x);
    }
    count = 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
};

// Deferred appends of a wave (fused append): lane r holds, for the r-th stream end the wave has
// walked, the granule of the block that takes the new token, the token's slot in that block and
// the segment.  The rows are written when the wave has finished its ranges (or the list is
// full): a store in the middle of the load pipeline would hold every later load back.
struct AppendList {
  int count, gran, slot, sig;
  __device__ AppendList() : count(0), gran(0), slot(0), sig(0) {}
  __device__ void add(int lane, int granule, int t, int sigma) {
    if (lane == count) {
      gran = granule;
      slot = t;
      sig = sigma;
    }
    ++count;
  }
};

// K row: D/32 pieces of 64 bytes, lanes [0, D/8) copy 16 bytes each.  V row: one 2-byte slot in
// each 8-byte token quad; lanes [0, D/2) read the 16 bytes that hold two dims of the quad,
// replace the token's two slots and store them back.
template <int D>
__device__ __forceinline__ void append_rows(const Params& p, AppendList& list, int lane) {
  for (int r = 0; r < list.count; ++r) {
    const int g = __builtin_amdgcn_readlane(list.gran, r);
    const int t = __builtin_amdgcn_readlane(list.slot, r);
    const int sigma = __builtin_amdgcn_readlane(list.sig, r);
    const size_t base = (size_t)g * (kBlock * D);
    const uint16_t* krow = p.k_new + (size_t)sigma * D;
    const uint16_t* vrow = p.v_new + (size_t)sigma * D;
    if (lane < D / 8)
      *reinterpret_cast<u32x4*>(p.k_pool_w + base + k_elem(t, lane * 8)) =
          *reinterpret_cast<const u32x4*>(krow + lane * 8);
    if (lane < D / 2) {
      uint16_t* quad = p.v_pool_w + base + v_elem(t & ~3, 2 * lane, D);  // dims 2*lane, 2*lane+1
      u32x4 x = *reinterpret_cast<const u32x4*>(quad);
      const uint32_t two = *reinterpret_cast<const uint32_t*>(vrow + 2 * lane);
      const int e = t & 3;
      const uint32_t keep = (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
      const int sh = (e & 1) * 16;
      const uint32_t d0 = (two & 0xFFFFu) << sh, d1 = (two >> 16) << sh;
      if (e < 2) {
        x.x = (x.x & keep) | d0;
        x.z = (x.z & keep) | d1;
      } else {
        x.y = (x.y & keep) | d0;
        x.w = (x.w & keep) | d1;
      }
      *reinterpret_cast<u32x4*>(quad) = x;
    }
  }
  list.count = 0;
}

// The records a wave has just copied to global memory are counted, one atomic per record, on
// their segments' counters; a segment whose count is complete (or that has a single run) is
// merged here and now, and its counter goes back to zero for the next launch.  The fences make
// the records of other waves (any compute die) visible to the wave that merges them.
template <int D>
__device__ __forceinline__ void arrive_and_merge(const Params& p, const float2* pml, const float* pacc,
                                        int count, int sigs, int lane) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  int2 info = make_int2(0, 0);
  int old = -1;
  if (lane < count) {
    info = p.seg_info[sigs];
    if (info.y > 1)
      old = __hip_atomic_fetch_add(p.seg_count + sigs, 1, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
  }
  unsigned long long mask =
      __builtin_amdgcn_ballot_w64(lane < count && (info.y == 1 || old == info.y - 1));
  if (mask == 0) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  while (mask) {
    const int r = __builtin_ctzll(mask);
    mask &= mask - 1;
    const int sigma = __builtin_amdgcn_readlane(sigs, r);
    const int slot0 = __builtin_amdgcn_readlane(info.x, r);
    const int n = __builtin_amdgcn_readlane(info.y, r);
    const int s = sigma / p.Hkv, h = sigma - s * p.Hkv;
    const size_t row = (size_t)(p.q_rows ? p.q_rows[s] : s) * p.Hq + (size_t)h * p.G;
    merge_segment<D>(pml, pacc, slot0, n, p.G, lane, p.out + row * D, p.lse ? p.lse + row : nullptr);
    if (n > 1 && lane == 0)
      __hip_atomic_store(p.seg_count + sigma, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <class Math>
__global__ __launch_bounds__(256, Math::kMinWavesPerSimd) void decode_kernel(
    Params p, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ header,
    const typename Math::Desc* __restrict__ desc, float2* __restrict__ pml,
    float* __restrict__ pacc) {
  typedef typename Math::Desc Desc;
  constexpr int NBUF = Math::kBuffers;
  constexpr int LA = NBUF + 1;  // descriptor look-ahead in steps
  constexpr int D = Math::kHeadDim;
  const int lane = threadIdx.x & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6));
  // The wave's first range: from the plan's table, or static range w of the layout.
  StepLayout lay = layout_of(0, 1, false);  // no pool unless the static layout says so
  int64_t x0 = 0;
  int nsteps = 0;
  bool idle = false;  // nothing to walk at all
  if (p.ranges_off > 0) {  // ranges of unequal length, balanced by the plan
    const int32_t* r = header + p.ranges_off;
    x0 = r[w];
    nsteps = r[w + 1] - r[w];
    idle = nsteps <= 0;
  } else {
    lay = p.n_steps >= 0 ? p.lay : layout_from_header(header);
    x0 = (int64_t)w * lay.Q;
    if (x0 < lay.n_main) nsteps = (int)min((int64_t)lay.Q, lay.n_main - x0);
    idle = nsteps <= 0 && lay.R == 0;
  }
  if constexpr (!Math::kSelfMerge) {
    if (idle) return;
  }
  int range = w;  // index of the range being walked: static range w, then pool ranges U + j
  const unsigned long long t_start = p.wave_clock ? wall_clock64() : 0;
  __shared__ float stash_mem[kWavesPerGroup][Math::kStashFloats];
  PartialStash stash(stash_mem[threadIdx.x >> 6], Math::kStashFloats, Math::columns(p), p.D, lane);
  Math math(lane, p);
  typename Math::State st;
  typename Math::Q qnext;
  typename Math::Regs ring[NBUF];
  AppendList appends;
  // Records leave the LDS buffer; with the merge by the last arriver their arrival is counted
  // right away, so that a segment is merged as soon as its last record is out.
  const auto flush_records = [&]() {
    const int count = stash.count;
    stash.flush(pml, pacc);
    if constexpr (Math::kSelfMerge) {
      if (count > 0) arrive_and_merge<D>(p, pml, pacc, count, stash.sigs, lane);
    }
  };
  // One step of the pipeline.  In the steady-state loop every step refills its ring slot
  // unconditionally: a load issued under a run-time condition makes the compiler's wait-count
  // bookkeeping assume it was not issued and wait for every younger load, which serialises
  // memory and arithmetic.  Refills past the end of the range are pointed at granule 0 of the
  // pools (always mapped, cache resident after the first touch) and never consumed.
#define VOX_STEP(I, B, REFILL)                                                             \
  {                                                                                        \
    const int i = (I);                                                                     \
    const Desc dcur = dq[0];                                                               \
    const int meta = Math::meta(dcur);                                                     \
    const int sigma = Math::sigma(dcur);                                                   \
    if (meta & kMetaFirst) {                                                               \
      math.reset(st);                                                                      \
      math.install_q(st, qnext);                                                           \
    }                                                                                      \
    if constexpr (Math::kFusedAppend) {                                                    \
      if (p.k_new && (meta & kMetaTail)) {                                                 \
        if (appends.count == kWave) append_rows<D>(p, appends, lane);                      \
        const int tn = (meta & kMetaTokMask) - 1; /* the newest token's place in the step */ \
        math.patch_new_token(ring[B], dcur);                                               \
        appends.add(lane, tn < kBlock ? Math::ga(dcur) : Math::gb(dcur), tn & (kBlock - 1), \
                    sigma);                                                                \
      }                                                                                    \
    }                                                                                      \
    math.compute(st, ring[B], dcur);                                                       \
    if (i + 1 < nsteps && (Math::meta(dq[1]) & kMetaFirst))                                \
      math.load_q(qnext, st, q, dq[1]);                                                    \
    if (REFILL) {                                                                          \
      const bool more = i + NBUF < nsteps;                                                 \
      math.template issue<true>(ring[B], k_pool, v_pool, more ? Math::ga(dq[NBUF]) : 0,    \
                                more ? Math::gb(dq[NBUF]) : 0);                            \
      if constexpr (Math::kFusedAppend) {                                                  \
        if (p.k_new && more && (Math::meta(dq[NBUF]) & kMetaTail))                         \
          math.issue_new_token(ring[B], dq[NBUF]);                                         \
      }                                                                                    \
    }                                                                                      \
    if (meta & kMetaLast) {                                                                \
      bool whole = false; /* the run is its whole segment: finished rows, no partial record */ \
      if constexpr (Math::kDirect) whole = (meta & kMetaWhole) != 0;                       \
      if (whole) {                                                                         \
        if constexpr (Math::kDirect) math.finish_rows(st, dcur);                           \
      } else if (stash.cap > 0) {                                                          \
        if constexpr (Math::kSelfMerge) {                                                  \
          if (stash.full()) flush_records();                                               \
        }                                                                                  \
        float* rec = stash.next(pml, pacc);                                                \
        math.finish(st, rec, rec + stash.gd);                                              \
        stash.commit(range + sigma, math.used_columns(dcur), sigma);                       \
      } else { /* record larger than the LDS buffer: straight to global memory */          \
        const size_t slot = (size_t)(range + sigma);                                       \
        math.finish(st, pacc + slot * stash.gd,                                            \
                    reinterpret_cast<float*>(pml + slot * Math::columns(p)));              \
      }                                                                                    \
    }                                                                                      \
    _Pragma("unroll") for (int k = 0; k < LA; ++k) dq[k] = dq[k + 1];                      \
    dq[LA] = dbase[min(i + 1 + LA, nsteps - 1)];                                           \
  }

  while (!idle) {
    if (nsteps > 0) {
      // Descriptors are wave-uniform: they are fetched with scalar loads LA steps ahead and
      // live in scalar registers.  dq[k] is the descriptor of step i + k.
      const Desc* dbase = desc + x0;
      Desc dq[LA + 1];
#pragma unroll
      for (int k = 0; k <= LA; ++k) dq[k] = dbase[min(k, nsteps - 1)];

      math.load_q(qnext, st, q, dq[0]);
      math.reset(st);
#pragma unroll
      for (int b = 0; b < NBUF; ++b) {
        const bool more = b < nsteps;
        math.template issue<true>(ring[b], k_pool, v_pool, more ? Math::ga(dq[b]) : 0,
                                  more ? Math::gb(dq[b]) : 0);
        if constexpr (Math::kFusedAppend) {
          if (p.k_new && more && (Math::meta(dq[b]) & kMetaTail))
            math.issue_new_token(ring[b], dq[b]);
        }
      }

      int i0 = 0;
      for (; i0 + NBUF <= nsteps; i0 += NBUF) {  // whole groups of NBUF steps, no conditions
#pragma unroll
        for (int b = 0; b < NBUF; ++b) VOX_STEP(i0 + b, b, true)
      }
#pragma unroll
      for (int b = 0; b < NBUF - 1; ++b)  // fewer than NBUF steps remain; their data is in flight
        if (i0 + b < nsteps) VOX_STEP(i0 + b, b, false)
    }
    // the next range comes from the pool, if there is one and it is not used up
    if (lay.R == 0) break;
    int j = 0;
    if (lane == 0) j = atomicAdd(p.pool_counter, 1);
    j = __builtin_amdgcn_readfirstlane(j);
    if (j >= lay.R) break;
    range = lay.U + j;
    x0 = lay.n_main + (int64_t)j * lay.P;
    nsteps = (int)min((int64_t)lay.P, lay.N - x0);
  }
#undef VOX_STEP
  if constexpr (Math::kFusedAppend) {
    if (appends.count > 0) append_rows<D>(p, appends, lane);
  }
  flush_records();
  if constexpr (Math::kSelfMerge) {
    // streams without tokens own no segment: their output rows are zeroed here
    if (!p.q_rows) {
      const int nwaves = gridDim.x * kWavesPerGroup;
      for (int s = w; s < p.S; s += nwaves) {
        if (p.lens[s] > 0) continue;
        float* row = p.out + (size_t)s * p.Hq * D;
        for (int x = lane; x < p.Hq * D; x += kWave) row[x] = 0.f;
        if (p.lse && lane < p.Hq) p.lse[(size_t)s * p.Hq + lane] = -INFINITY;
      }
    }
  }
  if (p.wave_clock && lane == 0 && !idle) {
    p.wave_clock[2 * (size_t)w] = t_start;
    p.wave_clock[2 * (size_t)w + 1] = wall_clock64();
  }
}

}  // namespace vox
