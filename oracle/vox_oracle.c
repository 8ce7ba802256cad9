/*
 * CPU oracle for the decode step's KV-cache operations.  TEST INFRASTRUCTURE
 * ONLY: it is called by tests/, by the smoke check and by the benchmark's
 * cpu_baseline leg; the product path never links, loads or calls it.  It shares
 * no code with the HIP library.
 *
 * What it computes is the plain definition of the operations the paper places
 * in the decode operation of the serving Worker (Section 3; Section 3.1 "LLM
 * Forward"; Section 3.1.1 attention backend).  The paper gives no formula for
 * them, so the definition is textbook softmax attention, one query row per
 * stream, read through a block table, written out in fp64 with no blocking,
 * fusion or reordering:
 *
 *   z_t = scale * sum_d q[d] * K[t][d],  p = softmax(z),  out = sum_t p_t V[t]
 *
 * bf16 inputs are widened exactly; `scale` arrives as the fp32 value the caller
 * passes to the library and is widened exactly too.
 *
 * Cache layout (the library ABI this oracle is the reference for):
 *   K element (blk,h,t,d) at (((blk*Hkv+h)*(D/32) + d/32)*B + t)*32 + d%32
 *   V element (blk,h,t,d) at (((blk*Hkv+h)*(B/4) + t/4)*D + d)*4 + t%4
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force dense attention in
 * numpy and in exact rational arithmetic on tiny inputs, single-key and
 * equal-score closed forms, block permutation invariance, NaN poisoning of
 * unread slots, power-of-two rescaling (bit-exact), score-shift invariance,
 * GQA-vs-MHA reduction, convexity, lse consistency.  Against values printed in
 * the paper: none exist for this path, so parity is unpinned in that sense.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_BLOCK (-2) /* a block id that must be read is outside [0,P) */
#define ORACLE_ERR_MEM (-3)

static double bf16_to_f64(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static size_t k_index(int Hkv, int D, int B, int64_t blk, int h, int t, int d) {
  return ((((size_t)blk * Hkv + h) * (size_t)(D / 32) + (size_t)(d / 32)) * B + t) * 32 + (d % 32);
}

static size_t v_index(int Hkv, int D, int B, int64_t blk, int h, int t, int d) {
  return ((((size_t)blk * Hkv + h) * (size_t)(B / 4) + (size_t)(t / 4)) * D + d) * 4 + (t % 4);
}

static int shape_ok(int S, int Hq, int Hkv, int D, int B, int P, int max_nb) {
  return S > 0 && Hq > 0 && Hkv > 0 && Hq % Hkv == 0 && D > 0 && D % 32 == 0 && B > 0 && B % 4 == 0 && P > 0 &&
         max_nb > 0;
}

/* Physical block of logical token t of stream s, or -1 if the table entry is invalid. */
static int64_t block_of(const int32_t* bt, int max_nb, int P, int B, int s, int t) {
  int j = t / B;
  if (j >= max_nb) return -1;
  int32_t blk = bt[(size_t)s * max_nb + j];
  return (blk < 0 || blk >= P) ? -1 : (int64_t)blk;
}

/* Append: position L_s - 1 of every active stream receives k_new / v_new bit for bit. */
int vox_oracle_kv_append(int S, int Hkv, int D, int B, int P, int max_nb, const uint16_t* k_new,
                         const uint16_t* v_new, uint16_t* k_pool, uint16_t* v_pool,
                         const int32_t* bt, const int32_t* lens) {
  if (!shape_ok(S, Hkv, Hkv, D, B, P, max_nb)) return ORACLE_ERR_ARG;
  for (int s = 0; s < S; ++s) {
    int L = lens[s];
    if (L < 0) return ORACLE_ERR_ARG;
    if (L == 0) continue;
    int p = L - 1;
    int64_t blk = block_of(bt, max_nb, P, B, s, p);
    if (blk < 0) return ORACLE_ERR_BLOCK;
    int t = p % B;
    for (int h = 0; h < Hkv; ++h)
      for (int d = 0; d < D; ++d) {
        size_t src = ((size_t)s * Hkv + h) * D + d;
        k_pool[k_index(Hkv, D, B, blk, h, t, d)] = k_new[src];
        v_pool[v_index(Hkv, D, B, blk, h, t, d)] = v_new[src];
      }
  }
  return ORACLE_OK;
}

/* Gather: rows row_offsets[s] + t of k_out / v_out ([rows][Hkv][D]) get token t of stream s. */
int vox_oracle_kv_gather(int S, int Hkv, int D, int B, int P, int max_nb, const uint16_t* k_pool,
                         const uint16_t* v_pool, const int32_t* bt, const int32_t* lens,
                         const int64_t* row_offsets, uint16_t* k_out, uint16_t* v_out) {
  if (!shape_ok(S, Hkv, Hkv, D, B, P, max_nb)) return ORACLE_ERR_ARG;
  for (int s = 0; s < S; ++s) {
    for (int t = 0; t < lens[s]; ++t) {
      int64_t blk = block_of(bt, max_nb, P, B, s, t);
      if (blk < 0) return ORACLE_ERR_BLOCK;
      for (int h = 0; h < Hkv; ++h)
        for (int d = 0; d < D; ++d) {
          size_t dst = (((size_t)row_offsets[s] + t) * Hkv + h) * D + d;
          k_out[dst] = k_pool[k_index(Hkv, D, B, blk, h, t % B, d)];
          v_out[dst] = v_pool[v_index(Hkv, D, B, blk, h, t % B, d)];
        }
    }
  }
  return ORACLE_OK;
}

/*
 * Attention of one query row over tokens [0, ctx) of stream s, kv head h: the definition above,
 * nothing else.  o receives D doubles; returns ORACLE_OK, ORACLE_ERR_BLOCK or ORACLE_ERR_MEM.
 */
static int attend(int Hkv, int D, int B, int P, int max_nb, float scale, const uint16_t* qrow,
                  const uint16_t* k_pool, const uint16_t* v_pool, const int32_t* bt, int s, int h,
                  int ctx, double* o, double* lse_out) {
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  if (ctx <= 0) {
    if (lse_out) *lse_out = -INFINITY;
    return ORACLE_OK;
  }
  double* z = (double*)malloc((size_t)ctx * sizeof(double));
  if (!z) return ORACLE_ERR_MEM;
  double zmax = -INFINITY;
  for (int t = 0; t < ctx; ++t) {
    int64_t blk = block_of(bt, max_nb, P, B, s, t);
    if (blk < 0) {
      free(z);
      return ORACLE_ERR_BLOCK;
    }
    double dot = 0.0;
    for (int d = 0; d < D; ++d)
      dot += bf16_to_f64(qrow[d]) * bf16_to_f64(k_pool[k_index(Hkv, D, B, blk, h, t % B, d)]);
    z[t] = (double)scale * dot;
    if (z[t] > zmax) zmax = z[t];
  }
  double denom = 0.0;
  for (int t = 0; t < ctx; ++t) {
    z[t] = exp(z[t] - zmax);
    denom += z[t];
  }
  for (int t = 0; t < ctx; ++t) {
    int64_t blk = block_of(bt, max_nb, P, B, s, t);
    double p = z[t] / denom;
    for (int d = 0; d < D; ++d)
      o[d] += p * bf16_to_f64(v_pool[v_index(Hkv, D, B, blk, h, t % B, d)]);
  }
  if (lse_out) *lse_out = zmax + log(denom);
  free(z);
  return ORACLE_OK;
}

/*
 * Decode for streams [s0, s0+ns): out is fp64 [ns][Hq][D], lse fp64 [ns][Hq] (may be NULL).
 * Inactive streams (L == 0) give out = 0, lse = -inf.
 */
int vox_oracle_paged_decode(int S, int Hq, int Hkv, int D, int B, int P, int max_nb, float scale,
                            const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                            const int32_t* bt, const int32_t* lens, int s0, int ns, double* out,
                            double* lse) {
  if (!shape_ok(S, Hq, Hkv, D, B, P, max_nb) || s0 < 0 || ns < 0 || s0 + ns > S)
    return ORACLE_ERR_ARG;
  const int G = Hq / Hkv;
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int item = 0; item < ns * Hq; ++item) {
    const int s = s0 + item / Hq, i = item % Hq;
    const int rc = attend(Hkv, D, B, P, max_nb, scale, q + ((size_t)s * Hq + i) * D, k_pool,
                          v_pool, bt, s, i / G, lens[s], out + (size_t)item * D,
                          lse ? lse + item : NULL);
    if (rc != ORACLE_OK) {
#pragma omp atomic write
      status = rc;
    }
  }
  return status;
}

/*
 * Multi-token step (prompt prefill, chunked admission, detokenizer chunks): stream s brings
 * n_s = q_offsets[s+1] - q_offsets[s] new tokens, rows q_offsets[s] .. of the packed arrays,
 * occupying positions L_s - n_s .. L_s - 1 (L_s counts them).  Query j of the stream attends
 * causally: to tokens [0, L_s - n_s + j].
 */
int vox_oracle_kv_append_multi(int S, int Hkv, int D, int B, int P, int max_nb,
                               const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                               uint16_t* v_pool, const int32_t* bt, const int32_t* lens,
                               const int32_t* q_offsets) {
  if (!shape_ok(S, Hkv, Hkv, D, B, P, max_nb)) return ORACLE_ERR_ARG;
  for (int s = 0; s < S; ++s) {
    const int n = q_offsets[s + 1] - q_offsets[s];
    if (n < 0 || n > lens[s]) return ORACLE_ERR_ARG;
    for (int j = 0; j < n; ++j) {
      const int pos = lens[s] - n + j;
      int64_t blk = block_of(bt, max_nb, P, B, s, pos);
      if (blk < 0) return ORACLE_ERR_BLOCK;
      for (int h = 0; h < Hkv; ++h)
        for (int d = 0; d < D; ++d) {
          size_t src = (((size_t)q_offsets[s] + j) * Hkv + h) * D + d;
          k_pool[k_index(Hkv, D, B, blk, h, pos % B, d)] = k_new[src];
          v_pool[v_index(Hkv, D, B, blk, h, pos % B, d)] = v_new[src];
        }
    }
  }
  return ORACLE_OK;
}

/* out fp64 [Tq][Hq][D], lse fp64 [Tq][Hq] (may be NULL), Tq = q_offsets[S]. */
int vox_oracle_paged_prefill(int S, int Hq, int Hkv, int D, int B, int P, int max_nb, float scale,
                             const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                             const int32_t* bt, const int32_t* lens, const int32_t* q_offsets,
                             double* out, double* lse) {
  if (!shape_ok(S, Hq, Hkv, D, B, P, max_nb)) return ORACLE_ERR_ARG;
  const int G = Hq / Hkv;
  for (int s = 0; s < S; ++s) {
    const int n = q_offsets[s + 1] - q_offsets[s];
    if (n < 0 || n > lens[s]) return ORACLE_ERR_ARG;
  }
  const int Tq = q_offsets[S];
  int* row_stream = (int*)malloc(((size_t)Tq + 1) * sizeof(int));
  if (!row_stream) return ORACLE_ERR_MEM;
  for (int s = 0; s < S; ++s)
    for (int r = q_offsets[s]; r < q_offsets[s + 1]; ++r) row_stream[r] = s;
  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int item = 0; item < Tq * Hq; ++item) {
    const int row = item / Hq, i = item % Hq, s = row_stream[row];
    const int n = q_offsets[s + 1] - q_offsets[s];
    const int ctx = lens[s] - n + (row - q_offsets[s]) + 1;
    const int rc = attend(Hkv, D, B, P, max_nb, scale, q + (size_t)item * D, k_pool, v_pool, bt,
                          s, i / G, ctx, out + (size_t)item * D, lse ? lse + item : NULL);
    if (rc != ORACLE_OK) {
#pragma omp atomic write
      status = rc;
    }
  }
  free(row_stream);
  return status;
}

/* Threads the decode loop would use (for reporting the baseline's core count). */
/*
 * Fused step input: rotary position embedding + split of the layer's packed Q/K/V rows +
 * append (the work the serving loop does between the QKV projection and the attention call;
 * Section 3.1.1 puts the whole LLM Forward stage on one captured fast path, so these small
 * steps are folded into the append).  The paper does not describe the backbone's position
 * encoding; the rotation is the published rotary embedding in the half-split convention of
 * the Llama / Qwen family its backbones come from:
 *
 *   for i < D/2:  y[i]       = x[i] * cos[pos][i]       - x[i + D/2] * sin[pos][i]
 *                 y[i + D/2] = x[i + D/2] * cos[pos][i] + x[i] * sin[pos][i]
 *
 * applied to every q head and every k head of stream s at pos = L_s - 1; v is not rotated.
 * The result is a bf16 bit pattern, i.e. floating point decides a 16-bit code, so the
 * arithmetic is fixed and is the library's: both products and their sum/difference are
 * separate fp32 operations, each rounded to nearest (no fused multiply-add; this file is
 * compiled with -ffp-contract=off), followed by one round-to-nearest-even to bf16.  cos / sin
 * arrive as fp32 tables [positions][D/2] made by the caller.
 *   qkv   : [S][Hq + 2*Hkv][D] bf16 (q heads, then k heads, then v heads)
 *   q_out : [S][Hq][D] bf16; rows of streams with L_s = 0 are left untouched
 * Pins (tests/test_oracle_rope_pins.py): quarter-turn worked example, identity at angle 0,
 * agreement with an fp64 evaluation to half a bf16 ulp, relative-position property of the
 * rotated dot product, v and untouched slots bit-identical, equality with kv_append when the
 * angle is 0.
 */
static float bf16_to_f32(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

static uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static void rotate_head(int D, const uint16_t* x, const float* c, const float* s, uint16_t* y) {
  int half = D / 2;
  for (int i = 0; i < half; ++i) {
    float a = bf16_to_f32(x[i]), b = bf16_to_f32(x[i + half]);
    float ac = a * c[i], bs = b * s[i], bc = b * c[i], as = a * s[i];
    y[i] = f32_to_bf16_rne(ac - bs);
    y[i + half] = f32_to_bf16_rne(bc + as);
  }
}

int vox_oracle_rope_append(int S, int Hq, int Hkv, int D, int B, int P, int max_nb,
                           const uint16_t* qkv, const float* rope_cos, const float* rope_sin,
                           int rope_positions, uint16_t* q_out, uint16_t* k_pool,
                           uint16_t* v_pool, const int32_t* bt, const int32_t* lens) {
  if (!shape_ok(S, Hq, Hkv, D, B, P, max_nb) || D % 2 || D > 1024) return ORACLE_ERR_ARG;
  int heads = Hq + 2 * Hkv;
  for (int s = 0; s < S; ++s) {
    int L = lens[s];
    if (L < 0) return ORACLE_ERR_ARG;
    if (L == 0) continue;
    int p = L - 1;
    if (p >= rope_positions) return ORACLE_ERR_ARG;
    int64_t blk = block_of(bt, max_nb, P, B, s, p);
    if (blk < 0) return ORACLE_ERR_BLOCK;
    int t = p % B;
    const float* c = rope_cos + (size_t)p * (D / 2);
    const float* sn = rope_sin + (size_t)p * (D / 2);
    const uint16_t* row = qkv + (size_t)s * heads * D;
    for (int i = 0; i < Hq; ++i) rotate_head(D, row + (size_t)i * D, c, sn, q_out + ((size_t)s * Hq + i) * D);
    for (int h = 0; h < Hkv; ++h) {
      uint16_t k_rot[1024];
      rotate_head(D, row + (size_t)(Hq + h) * D, c, sn, k_rot);
      const uint16_t* v = row + (size_t)(Hq + Hkv + h) * D;
      for (int d = 0; d < D; ++d) {
        k_pool[k_index(Hkv, D, B, blk, h, t, d)] = k_rot[d];
        v_pool[v_index(Hkv, D, B, blk, h, t, d)] = v[d];
      }
    }
  }
  return ORACLE_OK;
}

/* Number of OpenMP threads later calls may use (n < 1: the runtime's default). */
void vox_oracle_set_num_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n < 1 ? omp_get_num_procs() : n);
#else
  (void)n;
#endif
}

int vox_oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
