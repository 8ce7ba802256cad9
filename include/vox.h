/*
 * libvox: batched decode-step attention for SpeechLM serving on MI355X (gfx950).
 *
 * The operations are the two KV-cache touching pieces of the decode operation a
 * serving Worker executes for a batch of concurrent streams (paper Section 3,
 * "Worker ... prefill/decode/detokenize"; Section 3.1 "LLM Forward"; Section
 * 3.1.1 names the attention backend as the optimised part of that stage):
 *   1. append the K/V rows of the token just generated to a paged KV cache,
 *   2. attend, for each stream, its single new query over its whole cached
 *      context (grouped-query attention, one query row per stream).
 * The paper fixes neither layout nor kernel design; both are defined here.
 *
 * Conventions
 *   S    num_streams            Hq  num_q_heads      Hkv num_kv_heads
 *   G    Hq / Hkv  (q head i reads kv head i / G;  1 <= G <= 8)
 *   D    head_dim in {64, 128}  B   block_size == 16 tokens
 *   P    num_blocks in each pool
 *   L_s  context_lens[s]: tokens of stream s INCLUDING the one appended this
 *        step.  L_s == 0 marks a padded / inactive slot.
 *
 * KV-cache layout (part of the ABI, bf16 elements, two separate pools):
 *   K pool, element (blk, h, t, d), t in [0,B), d in [0,D):
 *       (((blk*Hkv + h)*(D/32) + d/32)*B + t)*32 + d%32
 *     i.e. [P][Hkv][D/32][B][32]: a token's row is D/32 pieces of 64 bytes.
 *   V pool, element (blk, h, t, d):
 *       (((blk*Hkv + h)*(B/4) + t/4)*D + d)*4 + t%4
 *     i.e. [P][Hkv][B/4][D][4]: four consecutive tokens of one dim are adjacent.
 *   Both serve the matrix-core operand shapes directly (8 consecutive dims of a
 *   token for QK^T, 4 consecutive tokens of a dim for PV) while an appended
 *   token touches only D/32 + D/16 cache lines of its block.
 *   Each (blk, h) pair is one contiguous granule of B*D*2 bytes in either pool.
 *   block_tables is int32 [S][max_blocks_per_stream]; logical token t of
 *   stream s lives in physical block block_tables[s][t / B], slot t % B.
 *   Entries at or past ceil(L_s / B) are never read.  Slots t >= L_s of the
 *   last block and blocks owned by no stream are never read either, whatever
 *   bits they hold.
 *
 * Pointers are DEVICE pointers unless marked host.  The caller owns every
 * buffer; the library allocates nothing, keeps no state between calls, and
 * every call only enqueues work on `hip_stream` (a hipStream_t, may be NULL
 * for the default stream) and returns: no synchronisation, no host copies.
 * Contents of device-resident block_tables / context_lens are trusted (block
 * ids outside [0,P) or L_s > max_blocks_per_stream*B are undefined behaviour).
 * Row tensors (q, k_new, v_new, qkv, q_out), the pools, the rotary tables and
 * the fp32 outputs are read and written 16 bytes at a time: their base
 * addresses must be multiples of 16 (VOX_ERR_ARG otherwise); int32 / int64 /
 * float arrays of per-stream scalars need only their natural alignment.
 *
 * Every function returns VOX_OK (0) or a negative VOX_ERR_* code; the host-side
 * checks (null pointers, shape rules, workspace size) run before any launch.
 */
#ifndef VOX_H_
#define VOX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VOX_OK 0
#define VOX_ERR_NULL (-1)      /* a required pointer is NULL */
#define VOX_ERR_SHAPE (-2)     /* S<=0, S>8192, Hq%Hkv!=0, G>8, D not in {64,128}, B!=16, P<=0, ... */
#define VOX_ERR_WORKSPACE (-3) /* workspace too small for the steps of this call */
#define VOX_ERR_HIP (-4)       /* a launch failed; hipGetLastError() still holds the cause */
#define VOX_ERR_ARG (-5)       /* a scalar argument is out of range, or a misaligned tensor */
#define VOX_ERR_SCRATCH (-6)   /* vox_paged_decode_static: the call needs more than the built-in scratch */

/* Size of the built-in scratch memory of vox_paged_decode_static (per GPU, held until the process ends). */
#define VOX_STATIC_SCRATCH_BYTES (64u << 20)

/* Which decode kernel family runs; both give results within the same tolerance. */
#define VOX_PATH_AUTO 0 /* the library's choice (MFMA) */
#define VOX_PATH_MFMA 1 /* QK^T and PV on bf16 matrix cores, P split into hi+lo bf16 */
#define VOX_PATH_VALU 2 /* fp32 vector ALU only; kept as the measured alternative */

typedef struct {
  int32_t num_streams;           /* S, may include padded slots with L_s == 0 */
  int32_t num_q_heads;           /* Hq */
  int32_t num_kv_heads;          /* Hkv */
  int32_t head_dim;              /* D */
  int32_t block_size;            /* B, must be 16 */
  int32_t num_blocks;            /* P */
  int32_t max_blocks_per_stream; /* row stride of block_tables */
  float scale;                   /* softmax scale applied to the fp32 dot product */
  int32_t decode_path;           /* VOX_PATH_* */
  int32_t split_waves;           /* split-K: number of waves the context steps of all streams
                                    are dealt to; 0 = one per wave the chip keeps resident
                                    (1024), the balanced single round */
} vox_shape_t;

/*
 * KV append (first half of the decode step: the new token's K/V rows enter the
 * cache before the query attends to them).  For every stream s with L_s > 0:
 * p = L_s - 1, blk = block_tables[s][p / B], t = p % B, and for every kv head h
 * and dim d the bf16 bit pattern k_new[s][h][d] is copied to K-pool element
 * (blk, h, t, d), v_new likewise to the V pool.  Nothing else is written.
 *   k_new, v_new : [S][Hkv][D] bf16, read only
 *   k_pool,v_pool: layouts above, modified in place
 */
int vox_kv_append(const vox_shape_t* shape, const void* k_new, const void* v_new, void* k_pool,
                  void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                  void* hip_stream);

/*
 * Block gather (the paged read the decode kernels perform, exposed on its own so
 * it can be checked bit for bit and used to export a stream's cache): for every
 * stream s and t < L_s, row row_offsets[s] + t of k_out / v_out ([rows][Hkv][D]
 * bf16, row-major) receives the K / V row of logical token t.
 *   row_offsets : int64 [S] device; rows of different streams must not overlap.
 */
int vox_kv_gather(const vox_shape_t* shape, const void* k_pool, const void* v_pool,
                  const int32_t* block_tables, const int32_t* context_lens,
                  const int64_t* row_offsets, void* k_out, void* v_out, void* hip_stream);

/*
 * Workspace for vox_paged_decode / vox_decode_step: split-K step descriptors and
 * the partial (max, sum, accumulator) records.  The returned size is enough for
 * any context_lens the shape admits (every stream at max_blocks_per_stream); a
 * smaller workspace is accepted when context_lens_host shows that the actual
 * number of 32-token steps fits.  Returns 0 on a bad shape.  The workspace must
 * be 256-byte aligned; its contents are scratch.
 */
size_t vox_paged_decode_workspace_bytes(const vox_shape_t* shape);

/*
 * Paged grouped-query attention decode (second half of the decode step).  For
 * every stream s with L = L_s > 0 and q head i (kv head h = i / G):
 *   z_t  = scale * sum_d q[s][i][d] * K(s,h,t,d)          t in [0, L)
 *   p    = softmax(z)
 *   out[s][i][:] = sum_t p_t * V(s,h,t,:)
 *   lse[s][i]    = log(sum_t exp(z_t))                     (natural log)
 * where K(s,h,t,d) / V(...) are read through block_tables.  Streams with
 * L_s == 0 get out = 0 and lse = -inf.  Inputs are bf16, accumulation fp32.
 *   q                 : [S][Hq][D] bf16
 *   context_lens_host : HOST copy of context_lens or NULL.  When given it must
 *                       equal the device array: the workspace check, the
 *                       planning grid, the number of attention waves that get
 *                       a range and the layout of the step axis the kernels
 *                       work from are then taken from it (this saves every
 *                       wave a dependent load).  With NULL all of that comes
 *                       from the device array and the shape's bounds, and no
 *                       launch depends on the lengths.
 *                       Graph capture: a captured call is replayed when the
 *                       device lengths may have changed, so while hip_stream
 *                       is being captured the host copy is IGNORED (treated
 *                       as NULL; the workspace must then have the full size
 *                       of vox_paged_decode_workspace_bytes).  A replay reads
 *                       context_lens and block_tables afresh and is correct
 *                       for any lengths the shape admits.  The same holds for
 *                       vox_decode_step and vox_decode_step_rope.
 *   out               : [S][Hq][D] fp32
 *   lse               : [S][Hq] fp32 or NULL
 * Split-K: the 32-token steps of all (stream, kv head) pairs are laid on one
 * axis and cut into ranges: equal ones, one per wave, plus (for long axes) a
 * pool of short ones that waves take as they finish; each run of a pair inside
 * a range leaves a partial softmax state in the workspace and a merge kernel
 * combines them.
 */
int vox_paged_decode(const vox_shape_t* shape, const void* q, const void* k_pool,
                     const void* v_pool, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* context_lens_host, float* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * vox_paged_decode for callers that cannot provide device memory beyond inputs and outputs and
 * must not allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as vox_paged_decode, without the workspace:
 * descriptors and partial records go to a built-in device array of VOX_STATIC_SCRATCH_BYTES
 * (64 MiB) that each GPU the library runs on holds until the process ends.  The call allocates
 * nothing and frees nothing.  Its very first use on a device looks up that device's copy of the
 * array (hipGetSymbolAddress; make that first call outside graph capture).  The array used is
 * the current device's (hipGetDevice): hip_stream must belong to the current device, as for
 * every launch.
 * Size limit: the call needs what vox_paged_decode_workspace_bytes(shape) reports (or, with
 * context_lens_host outside capture, the smaller amount the actual 32-token steps need); when
 * that exceeds VOX_STATIC_SCRATCH_BYTES it returns VOX_ERR_SCRATCH and launches nothing
 * (512 streams x 8192 tokens x 8 kv heads of head_dim 128 still fit without host lengths).
 * Every call on a GPU shares that GPU's array, which keeps the previous call's contents: the
 * planning kernel rewrites everything a call reads (header, pool counters, descriptors, step
 * prefix) before it is read, so nothing needs clearing between calls, but two calls whose
 * execution overlaps on one GPU (different streams, or concurrent graph launches) race on it.
 */
int vox_paged_decode_static(const vox_shape_t* shape, const void* q, const void* k_pool,
                            const void* v_pool, const int32_t* block_tables,
                            const int32_t* context_lens, const int32_t* context_lens_host,
                            float* out, float* lse, void* hip_stream);

/*
 * Measurement aid: vox_paged_decode that also records two caller-created hipEvent_t on
 * hip_stream, one immediately before and one immediately after the split-K attention kernel
 * (the launch that reads the KV cache), so its duration can be read with
 * hipEventElapsedTime.  Either event may be NULL.  wave_clock, when not NULL, is a device
 * array of 2 * W uint64 (W = split_waves, 1024 by default): wave w of the attention kernel
 * stores the chip's constant-rate clock (100 MHz) at its start and end in entries 2w, 2w+1;
 * entries of waves without work are left untouched.
 */
int vox_paged_decode_profiled(const vox_shape_t* shape, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* block_tables,
                              const int32_t* context_lens, const int32_t* context_lens_host,
                              float* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream, void* event_before, void* event_after,
                              uint64_t* wave_clock);

/*
 * Measurement aid: reads `bytes` (a multiple of 16) of device memory at buf once with the
 * attention kernel's memory pipeline and none of its arithmetic (one wave per SIMD, contiguous
 * shares, 16 KB steps of 16-byte streaming loads, three steps in flight per wave), and xors
 * one word per workgroup into sink (device, at least 8192 * 4 bytes, zeroed by the caller):
 * the streaming-read rate this chip reaches when nothing else is in the way.
 */
int vox_read_probe(const void* buf, size_t bytes, void* sink, void* hip_stream);

/*
 * Whole decode step over `num_layers` backbone layers that share block_tables
 * and context_lens (one allocation per stream, a pool pair per layer): for
 * l = 0..num_layers-1 in order, vox_kv_append then vox_paged_decode on layer l's
 * buffers.  The split-K step descriptors are built once and reused by every layer.
 * q, k_new, v_new, k_pool, v_pool, out are HOST arrays of num_layers device
 * pointers with the per-layer shapes documented above.
 */
int vox_decode_step(const vox_shape_t* shape, int32_t num_layers, const void* const* q,
                    const void* const* k_new, const void* const* v_new, void* const* k_pool,
                    void* const* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                    const int32_t* context_lens_host, float* const* out, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/*
 * The same step one layer at a time, for a backbone whose other kernels (projections, MLP) run
 * between the attention calls of consecutive layers (paper Section 3.1, LLM Forward: the
 * attention backend is called once per layer).  vox_decode_plan builds the split-K step
 * descriptors of this step's block_tables / context_lens once; vox_decode_layer then runs
 * vox_kv_append (skipped when k_new and v_new are both NULL) and the attention of one layer on
 * that plan.  `layer` in [0, 4096) names the layer (each has its own counter of the shared
 * range pool, set to zero by the plan): within one step, call every layer index at most once
 * after the plan.  Shape, block_tables, context_lens, context_lens_host, workspace and stream
 * must be the ones given to vox_decode_plan, and the workspace must not be used by anything
 * else between the plan and the step's last layer.  Results equal vox_decode_step's bit for
 * bit; lse may be NULL.  Graph capture: as for vox_paged_decode (the host copy is ignored).
 */
int vox_decode_plan(const vox_shape_t* shape, const int32_t* block_tables,
                    const int32_t* context_lens, const int32_t* context_lens_host, void* workspace,
                    size_t workspace_bytes, void* hip_stream);
int vox_decode_layer(const vox_shape_t* shape, int32_t layer, const void* q, const void* k_new,
                     const void* v_new, void* k_pool, void* v_pool, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* context_lens_host, float* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Fused step input (the paper puts the whole LLM Forward stage on one captured fast path,
 * Section 3.1.1, so the small steps between the QKV projection and the attention call are
 * folded into the append): rotary position embedding of q and k, split of the packed rows,
 * append of k and v.  For every stream with L_s > 0, at position pos = L_s - 1:
 *     i < D/2:  y[i]       = x[i] * cos[pos][i]       - x[i + D/2] * sin[pos][i]
 *               y[i + D/2] = x[i + D/2] * cos[pos][i] + x[i] * sin[pos][i]
 * for each q head (result to q_out) and each k head (result into the cache); v heads are copied
 * unrotated.  Arithmetic: fp32 products and sum as separate roundings, then round to nearest
 * even to bf16; the result is bit-reproducible.
 *   qkv       : [S][Hq + 2*Hkv][D] bf16 device: q heads, then k heads, then v heads
 *   rope_cos, rope_sin : fp32 device [rope_positions][D/2]; rope_positions must be at least
 *               max_blocks_per_stream * 16 (else VOX_ERR_ARG): the tables are indexed from
 *               device-side lengths
 *   q_out     : [S][Hq][D] bf16 device; rows of streams with L_s = 0 are left untouched
 * vox_decode_step_rope is vox_decode_step with this in place of the plain append: layer l
 * reads qkv[l], writes q_rot[l] (which the layer's attention then reads) and its pools; q_rot
 * entries may all name one buffer, since a layer's attention has finished before the next
 * layer's rows are written.
 */
int vox_rope_append(const vox_shape_t* shape, const void* qkv, const float* rope_cos,
                    const float* rope_sin, int32_t rope_positions, void* q_out, void* k_pool,
                    void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                    void* hip_stream);
int vox_decode_step_rope(const vox_shape_t* shape, int32_t num_layers, const void* const* qkv,
                         const float* rope_cos, const float* rope_sin, int32_t rope_positions,
                         void* const* q_rot, void* const* k_pool, void* const* v_pool,
                         const int32_t* block_tables, const int32_t* context_lens,
                         const int32_t* context_lens_host, float* const* out, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/*
 * Multi-token step: the prefill operation of the Worker (paper Section 3) and every other case
 * where a stream brings several new tokens at once: chunked admission of a prompt during the
 * startup phase (Section 3.2.1), or a detokenizer that keeps attention caches per request and
 * runs on chunks of tokens (Section 3.1, Postprocess).  Stream s brings
 * n_s = q_offsets[s+1] - q_offsets[s] tokens, rows q_offsets[s].. of the packed arrays, at
 * positions L_s - n_s .. L_s - 1 (L_s = context_lens[s] counts them; 0 <= n_s <= L_s).
 *
 * vox_kv_append_multi copies k_new / v_new ([total_q][Hkv][D] bf16) into those positions.
 * vox_paged_prefill computes, for query row r = q_offsets[s] + j and q head i,
 *     out[r][i][:] = softmax(scale * q[r][i] . K(s, i/G, 0 .. L_s - n_s + j)) V(...)
 * i.e. causal attention over the paged context (row j sees itself and everything before).
 *   q                 : [total_q][Hq][D] bf16;  out: [total_q][Hq][D] fp32;  lse: [total_q][Hq] or NULL
 *   q_offsets         : int32 [S+1] device, q_offsets[0] == 0
 *   context_lens_host, q_offsets_host : HOST copies, both required (the scheduler that admits
 *                       a prompt knows its length); sizes of the launches come from them
 *                       (a captured vox_paged_prefill therefore replays correctly only
 *                       while the device arrays still hold these values)
 * With no query rows at all (total_q == 0) both calls return VOX_OK and touch nothing.
 * vox_paged_prefill_workspace_bytes(shape, total_q) is enough for any lengths the shape
 * admits; a smaller workspace is accepted when the actual step count fits.
 * A batch may mix decoding streams (n_s = 1) with prompts and chunks, as during admission
 * (Section 3.2.1): when many streams bring exactly one token (32 or more, with 32 768 or more
 * 32-token steps between them, counted over all kv heads) those are computed by the kernels of
 * vox_paged_decode and the others by the multi-token kernels, in the same call and with the
 * same results; the workspace size above has room for both (with a smaller workspace every
 * stream takes the multi-token kernels).
 */
size_t vox_paged_prefill_workspace_bytes(const vox_shape_t* shape, int32_t total_q);
int vox_kv_append_multi(const vox_shape_t* shape, const void* k_new, const void* v_new,
                        void* k_pool, void* v_pool, const int32_t* block_tables,
                        const int32_t* context_lens, const int32_t* q_offsets, int32_t total_q,
                        void* hip_stream);
int vox_paged_prefill(const vox_shape_t* shape, const void* q, const void* k_pool,
                      const void* v_pool, const int32_t* block_tables,
                      const int32_t* context_lens, const int32_t* q_offsets,
                      const int32_t* context_lens_host, const int32_t* q_offsets_host,
                      float* out, float* lse, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/*
 * The multi-token step for a backbone that calls the attention once per layer (Section 3
 * "LLM Forward": every layer has its own cache, all layers share lengths, offsets and block
 * tables).  vox_prefill_plan does, once per step, everything of vox_paged_prefill that depends
 * only on those: tiles, wave ranges and step descriptors (and, for a mixed batch, the plan of
 * its decode part), left in the workspace.  vox_prefill_layer then runs one layer on that plan:
 * vox_kv_append_multi of k_new / v_new when they are given (both or neither), the attention
 * kernels and the merge; plan + layer give vox_paged_prefill's results bit for bit.  The host
 * copies, the shape and workspace_bytes must be the ones the plan was made with (the layer call
 * derives the same workspace map and the same split of a mixed batch from them); the plan stays
 * valid until the workspace is written by something else.  layer (0 <= layer < 4096) selects
 * the scheduling counter the decode part of a mixed batch uses, as in vox_decode_layer.
 */
int vox_prefill_plan(const vox_shape_t* shape, const int32_t* block_tables,
                     const int32_t* context_lens, const int32_t* q_offsets,
                     const int32_t* context_lens_host, const int32_t* q_offsets_host,
                     void* workspace, size_t workspace_bytes, void* hip_stream);
int vox_prefill_layer(const vox_shape_t* shape, int32_t layer, const void* q, const void* k_new,
                      const void* v_new, void* k_pool, void* v_pool, const int32_t* block_tables,
                      const int32_t* context_lens, const int32_t* q_offsets,
                      const int32_t* context_lens_host, const int32_t* q_offsets_host, float* out,
                      float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Measurement aid: vox_paged_prefill that also records two caller-created hipEvent_t on
 * hip_stream around the multi-token attention kernel (the launch that reads the KV cache; in a
 * mixed batch the two launches that do, decode kernel first).
 * Either event may be NULL; with no query rows at all nothing is launched or recorded.
 */
int vox_paged_prefill_profiled(const vox_shape_t* shape, const void* q, const void* k_pool,
                               const void* v_pool, const int32_t* block_tables,
                               const int32_t* context_lens, const int32_t* q_offsets,
                               const int32_t* context_lens_host, const int32_t* q_offsets_host,
                               float* out, float* lse, void* workspace, size_t workspace_bytes,
                               void* hip_stream, void* event_before, void* event_after);

/*
 * Sampling step (paper Section 3.1 "Sampling"; per-model settings in Appendix A): logits to the
 * next token of every stream, with repetition penalty, temperature, top-k and top-p.  For one
 * stream with logits z[V], recent tokens H (the row of `history`), uniform u in [0,1):
 *   1. z'_v = z_v / r if z_v > 0 else z_v * r for every v in H (once each; r = 1: off)
 *   2. y_v = z'_v / T                         (T <= 0: greedy, the first token of the order)
 *   3. order: descending y, ties by ascending token id
 *   4. top-k: the first k of the order (k <= 0 or k >= V: all)
 *   5. top-p: shortest prefix whose softmax weight reaches top_p of the kept total (>= 1: all)
 *   6. the first token of the prefix whose cumulative weight exceeds u * (weight of the prefix)
 * The arithmetic is fixed (single fp32 operations in a stated order, integer softmax weights
 * 2^40 * exp(y - max) from a fixed polynomial, integer cumulative sums), so the token is
 * reproducible bit for bit and independent of scheduling; the source states it step by step.
 *   logits   : fp32 device [num_streams][vocab], finite values; vocab <= 262144
 *   params   : device [num_streams]
 *   history  : int32 device [num_streams][window], ids outside [0, vocab) are empty slots;
 *              may be NULL when window == 0
 *   uniforms : fp32 device [num_streams], each in [0, 1)
 *   tokens   : int32 device [num_streams] (out);  kept: int32 device [num_streams] or NULL (out,
 *              size of the final prefix)
 * Nothing is allocated and no workspace is needed.
 */
typedef struct {
  float temperature;
  float top_p;
  float repetition_penalty;
  int32_t top_k;
} vox_sampling_t;

int vox_sample(int32_t num_streams, int32_t vocab, const float* logits,
               const vox_sampling_t* params, const int32_t* history, int32_t window,
               const float* uniforms, int32_t* tokens, int32_t* kept, void* hip_stream);

/*
 * Verification aid for vox_sample: for every token of every stream the distance
 * d = max_v y_v - y_v (fp32) and the integer softmax weight the draw uses, so that the fixed
 * arithmetic can be compared element by element.  d_out: fp32 device [num_streams][vocab];
 * w_out: uint64 device [num_streams][vocab].
 */
int vox_sample_weights(int32_t num_streams, int32_t vocab, const float* logits,
                       const vox_sampling_t* params, const int32_t* history, int32_t window,
                       float* d_out, uint64_t* w_out, void* hip_stream);

/* Static, never-NULL description of a return code. */
const char* vox_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* VOX_H_ */
