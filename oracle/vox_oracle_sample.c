/*
 * CPU oracle for the sampling step.  TEST INFRASTRUCTURE ONLY: called by tests/, the smoke
 * check and the benchmark's cpu_baseline leg; the product path never links, loads or calls it,
 * and it shares no code with the HIP library.
 *
 * The paper's Sampling stage (Section 3.1, "Sampling") turns the backbone's logits into the
 * next token with the standard algorithms: temperature, top-k, top-p and an optional
 * repetition penalty (Appendix A lists the per-model settings: temperature 0.6-0.8, top-p
 * 0.8-0.95, top-k 50, penalty 1.05-1.3).  It gives no formulas; the definition taken here, in
 * the order the common logits-processor chains apply them, for one stream with logits z[V],
 * window of recent tokens H, uniform u in [0,1):
 *
 *   1. penalty r:      z'_v = z_v / r if z_v > 0 else z_v * r   for every v in H (once each)
 *   2. temperature T:  y_v = z'_v / T                           (T <= 0: greedy, y = z')
 *   3. order:          descending y, ties by ascending token id
 *   4. top-k:          keep the first k of the order (k <= 0 or k >= V: all)
 *   5. top-p:          with softmax weights over the kept tokens, keep the shortest prefix
 *                      whose weight reaches top_p of the kept total (top_p >= 1: all; at
 *                      least one token)
 *   6. draw:           the first token of the prefix whose cumulative weight exceeds
 *                      u * (weight of the prefix); greedy takes the first token of the order
 *
 * Floating point decides an integer here (the token), so the arithmetic is fixed, and it is the
 * library's: every step below is a single IEEE fp32 operation or exact integer arithmetic, in
 * an order stated once, so that both sides get the same token bit for bit.
 *   invT = 1 / T (fp32 division);  y = z' * invT (fp32);  m = max y;  d = m - y (fp32) >= 0
 *   order key: the bits of d (non-negative floats order like their bits), then the token id
 *   weight w(d): x = d * log2(e) (fp32); n = floor(x), f = x - n; p = degree-9 Taylor
 *     polynomial of 2^-f in Horner form with fused multiply-adds; q = trunc(p * 2^24);
 *     w = (q << 16) >> n as a 64-bit integer (0 for x >= 64): w(0) = 2^40, sums of 2^18 weights
 *     fit 64 bits, and all cumulative sums are exact integers
 *   top-p threshold: trunc(double(top_p) * double(kept total)), at least 1
 *   draw target:     trunc(double(u) * double(prefix total)); first cumulative sum > target
 * Pins (tests/test_oracle_sample_pins.py): w(d) against exp(-d) to 4e-7 relative; the
 * distribution of draws over a grid of u against the softmax probabilities; top-k / top-p sets
 * against a numpy fp64 evaluation on inputs with clear margins; greedy = argmax; penalty and
 * tie rules on hand-made cases; the rows of vox_oracle_sample_weights against a numpy fp32
 * evaluation of d bit for bit, against exp, and against the prefixes vox_oracle_sample keeps.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_MEM (-3)

typedef struct {
  float temperature, top_p, repetition_penalty;
  int32_t top_k;
} vox_oracle_sampling_t;

static uint32_t f32_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  return u;
}

/* 2^40 * exp(-d) in the fixed arithmetic described above. */
uint64_t vox_oracle_sample_weight(float d) {
  const float log2e = 0x1.715476p+0f;
  float x = d * log2e;
  if (!(x < 64.0f)) return 0; /* also NaN */
  float nf = floorf(x);
  int n = (int)nf;
  float f = x - nf;
  float p = -0x1.b5253ep-24f;
  p = fmaf(p, f, 0x1.62c022p-20f);
  p = fmaf(p, f, -0x1.ffcbfcp-17f);
  p = fmaf(p, f, 0x1.430912p-13f);
  p = fmaf(p, f, -0x1.5d87fep-10f);
  p = fmaf(p, f, 0x1.3b2ab6p-7f);
  p = fmaf(p, f, -0x1.c6b08ep-5f);
  p = fmaf(p, f, 0x1.ebfbe0p-3f);
  p = fmaf(p, f, -0x1.62e430p-1f);
  p = fmaf(p, f, 1.0f);
  uint64_t q = (uint64_t)(uint32_t)(p * 16777216.0f);
  return (q << 16) >> n;
}

typedef struct {
  uint32_t dkey;
  int32_t id;
} ranked_t;

static int by_rank(const void* a, const void* b) {
  const ranked_t *x = a, *y = b;
  if (x->dkey != y->dkey) return x->dkey < y->dkey ? -1 : 1;
  return x->id < y->id ? -1 : (x->id > y->id);
}

/* Steps 1-2 and the distance to the maximum for one stream: y, m, d as the header states. */
static float tempered_row(int V, const float* z, const vox_oracle_sampling_t prm,
                          const int32_t* hist, int window, unsigned char* seen, float* y) {
  memset(seen, 0, (size_t)V);
  for (int j = 0; j < window; ++j) {
    int32_t v = hist[j];
    if (v >= 0 && v < V) seen[v] = 1;
  }
  const float r = prm.repetition_penalty;
  const float invT = (prm.temperature > 0.0f) ? 1.0f / prm.temperature : 1.0f;
  float m = -INFINITY;
  for (int v = 0; v < V; ++v) {
    float zp = z[v];
    if (seen[v]) zp = zp > 0.0f ? zp / r : zp * r;
    y[v] = zp * invT;
    if (y[v] > m) m = y[v];
  }
  return m;
}

/* d [S][V] and weights [S][V] of every token (what the draw is made from). */
int vox_oracle_sample_weights(int S, int V, const float* logits,
                              const vox_oracle_sampling_t* params, const int32_t* history,
                              int window, float* d_out, uint64_t* w_out) {
  if (S <= 0 || V <= 0 || window < 0 || (window > 0 && !history)) return ORACLE_ERR_ARG;
  float* y = malloc((size_t)V * sizeof(float));
  unsigned char* seen = malloc((size_t)V);
  if (!y || !seen) {
    free(y); free(seen);
    return ORACLE_ERR_MEM;
  }
  for (int s = 0; s < S; ++s) {
    float m = tempered_row(V, logits + (size_t)s * V, params[s],
                           window ? history + (size_t)s * window : NULL, window, seen, y);
    for (int v = 0; v < V; ++v) {
      float d = m - y[v];
      d_out[(size_t)s * V + v] = d;
      w_out[(size_t)s * V + v] = vox_oracle_sample_weight(d);
    }
  }
  free(y); free(seen);
  return ORACLE_OK;
}

/*
 * logits [S][V] fp32; params [S]; history [S][window] (ids outside [0,V) are empty slots) or
 * NULL; uniforms [S]; tokens [S] out; kept [S] out or NULL (size of the final prefix).
 */
int vox_oracle_sample(int S, int V, const float* logits, const vox_oracle_sampling_t* params,
                      const int32_t* history, int window, const float* uniforms,
                      int32_t* tokens, int32_t* kept) {
  if (S <= 0 || V <= 0 || window < 0 || (window > 0 && !history)) return ORACLE_ERR_ARG;
  float* y = malloc((size_t)V * sizeof(float));
  ranked_t* order = malloc((size_t)V * sizeof(ranked_t));
  uint64_t* w = malloc((size_t)V * sizeof(uint64_t));
  unsigned char* seen = malloc((size_t)V);
  if (!y || !order || !w || !seen) {
    free(y); free(order); free(w); free(seen);
    return ORACLE_ERR_MEM;
  }
  for (int s = 0; s < S; ++s) {
    const float* z = logits + (size_t)s * V;
    const vox_oracle_sampling_t prm = params[s];
    /* 1. repetition penalty on the tokens of the window, once each; 2. temperature */
    const int greedy = !(prm.temperature > 0.0f);
    float m = tempered_row(V, z, prm, window ? history + (size_t)s * window : NULL, window, seen, y);
    /* 3. order by (d, id); weights */
    for (int v = 0; v < V; ++v) {
      float d = m - y[v];
      order[v].dkey = f32_bits(d);
      order[v].id = v;
    }
    qsort(order, (size_t)V, sizeof(ranked_t), by_rank);
    for (int i = 0; i < V; ++i) {
      float d;
      memcpy(&d, &order[i].dkey, sizeof d);
      w[i] = vox_oracle_sample_weight(d);
    }
    if (greedy) {
      tokens[s] = order[0].id;
      if (kept) kept[s] = 1;
      continue;
    }
    /* 4. top-k */
    int n = (prm.top_k <= 0 || prm.top_k >= V) ? V : prm.top_k;
    uint64_t total = 0;
    for (int i = 0; i < n; ++i) total += w[i];
    /* 5. top-p */
    if (prm.top_p < 1.0f) {
      uint64_t thr = (uint64_t)((double)prm.top_p * (double)total);
      if (thr < 1) thr = 1;
      uint64_t cum = 0;
      int j = 0;
      while (j < n) {
        cum += w[j++];
        if (cum >= thr) break;
      }
      n = j;
      total = cum;
    }
    /* 6. draw */
    uint64_t target = (uint64_t)((double)uniforms[s] * (double)total);
    uint64_t cum = 0;
    int pick = n - 1;
    for (int i = 0; i < n; ++i) {
      cum += w[i];
      if (cum > target) {
        pick = i;
        break;
      }
    }
    tokens[s] = order[pick].id;
    if (kept) kept[s] = n;
  }
  free(y); free(order); free(w); free(seen);
  return ORACLE_OK;
}
