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
#pragma once

#include "vox_common.hpp"

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
  int lane;

  __device__ PartialStash(float* mem_, int floats, int cols, int D, int lane_)
      : mem(mem_), rec(cols * (D + 2)), gd(cols * D), cap(floats / (cols * (D + 2))),
        count(0), slots(0), used(0), lane(lane_) {}

  // LDS area of the record being added (older records are stored first if the buffer is
  // full); the caller fills [col][d] at col*D + d and the (max, sum) pair of column col at
  // gd + 2*col, then calls commit().
  __device__ float* next(float2* __restrict__ pml, float* __restrict__ pacc) {
    if (count == cap) flush(pml, pacc);
    return mem + count * rec;
  }

  __device__ void commit(int slot, int used_cols) {
    if (lane == count) {
      slots = slot;
      used = used_cols;
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

template <class Math>
__global__ __launch_bounds__(256, Math::kMinWavesPerSimd) void decode_kernel(
    Params p, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ header,
    const typename Math::Desc* __restrict__ desc, float2* __restrict__ pml,
    float* __restrict__ pacc) {
  typedef typename Math::Desc Desc;
  constexpr int NBUF = Math::kBuffers;
  constexpr int LA = NBUF + 1;  // descriptor look-ahead in steps
  const int lane = threadIdx.x & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6));
  // The wave's first range: from the plan's table, or static range w of the layout.
  StepLayout lay = layout_of(0, 1, false);  // no pool unless the static layout says so
  int64_t x0 = 0;
  int nsteps = 0;
  if (p.ranges_off > 0) {  // ranges of unequal length, balanced by the plan
    const int32_t* r = header + p.ranges_off;
    x0 = r[w];
    nsteps = r[w + 1] - r[w];
    if (nsteps <= 0) return;
  } else {
    lay = p.n_steps >= 0 ? p.lay : layout_from_header(header);
    x0 = (int64_t)w * lay.Q;
    if (x0 < lay.n_main) nsteps = (int)min((int64_t)lay.Q, lay.n_main - x0);
    if (nsteps <= 0 && lay.R == 0) return;
  }
  int range = w;  // index of the range being walked: static range w, then pool ranges U + j
  const unsigned long long t_start = p.wave_clock ? wall_clock64() : 0;
  __shared__ float stash_mem[kWavesPerGroup][Math::kStashFloats];
  PartialStash stash(stash_mem[threadIdx.x >> 6], Math::kStashFloats, Math::columns(p), p.D, lane);
  Math math(lane, p);
  typename Math::State st;
  typename Math::Q qnext;
  typename Math::Regs ring[NBUF];
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
    math.compute(st, ring[B], dcur);                                                       \
    if (i + 1 < nsteps && (Math::meta(dq[1]) & kMetaFirst))                                \
      math.load_q(qnext, st, q, dq[1]);                                                    \
    if (REFILL) {                                                                          \
      const bool more = i + NBUF < nsteps;                                                 \
      math.template issue<true>(ring[B], k_pool, v_pool, more ? Math::ga(dq[NBUF]) : 0,    \
                                more ? Math::gb(dq[NBUF]) : 0);                            \
    }                                                                                      \
    if (meta & kMetaLast) {                                                                \
      bool whole = false; /* the run is its whole segment: finished rows, no partial record */ \
      if constexpr (Math::kDirect) whole = (meta & kMetaWhole) != 0;                       \
      if (whole) {                                                                         \
        if constexpr (Math::kDirect) math.finish_rows(st, dcur);                           \
      } else if (stash.cap > 0) {                                                          \
        float* rec = stash.next(pml, pacc);                                                \
        math.finish(st, rec, rec + stash.gd);                                              \
        stash.commit(range + sigma, math.used_columns(dcur));                              \
      } else { /* record larger than the LDS buffer: straight to global memory */          \
        const size_t slot = (size_t)(range + sigma);                                       \
        math.finish(st, pacc + slot * stash.gd,                                            \
                    reinterpret_cast<float*>(pml + slot * Math::columns(p)));              \
      }                                                                                    \
    }                                                                                      \
    _Pragma("unroll") for (int k = 0; k < LA; ++k) dq[k] = dq[k + 1];                      \
    dq[LA] = dbase[min(i + 1 + LA, nsteps - 1)];                                           \
  }

  for (;;) {
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
  stash.flush(pml, pacc);
  if (p.wave_clock && lane == 0) {
    p.wave_clock[2 * (size_t)w] = t_start;
    p.wave_clock[2 * (size_t)w + 1] = wall_clock64();
  }
}

}  // namespace vox
