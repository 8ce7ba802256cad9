/* Small driver that runs every oracle entry point on a seeded problem; built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitized.py to catch out-of-bounds
 * indexing and undefined behaviour in the oracle's C. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int vox_oracle_kv_append(int, int, int, int, int, int, const uint16_t*, const uint16_t*, uint16_t*,
                         uint16_t*, const int32_t*, const int32_t*);
int vox_oracle_kv_gather(int, int, int, int, int, int, const uint16_t*, const uint16_t*,
                         const int32_t*, const int32_t*, const int64_t*, uint16_t*, uint16_t*);
int vox_oracle_paged_decode(int, int, int, int, int, int, int, float, const uint16_t*,
                            const uint16_t*, const uint16_t*, const int32_t*, const int32_t*, int,
                            int, double*, double*);

int vox_oracle_kv_append_multi(int, int, int, int, int, int, const uint16_t*, const uint16_t*,
                               uint16_t*, uint16_t*, const int32_t*, const int32_t*,
                               const int32_t*);
int vox_oracle_paged_prefill(int, int, int, int, int, int, int, float, const uint16_t*,
                             const uint16_t*, const uint16_t*, const int32_t*, const int32_t*,
                             const int32_t*, double*, double*);
int vox_oracle_rope_append(int, int, int, int, int, int, int, const uint16_t*, const float*,
                           const float*, int, uint16_t*, uint16_t*, uint16_t*, const int32_t*,
                           const int32_t*);

typedef struct {
  float temperature, top_p, repetition_penalty;
  int32_t top_k;
} sampling_t;
int vox_oracle_sample(int, int, const float*, const sampling_t*, const int32_t*, int,
                      const float*, int32_t*, int32_t*);

static uint32_t state = 12345u;
static uint16_t rnd_bf16(void) { /* values in about [-2, 2) with a few mantissa bits */
  state = state * 1664525u + 1013904223u;
  int v = (int)((state >> 20) & 255) - 128;
  float f = (float)v / 64.0f;
  uint32_t u;
  __builtin_memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

int main(void) {
  enum { S = 5, Hq = 6, Hkv = 2, D = 64, B = 16, P = 23, MAXNB = 6 };
  const int32_t lens[S] = {1, 16, 17, 0, 96};
  int32_t bt[S * MAXNB];
  int next = P - 1; /* deal blocks from the top so the highest block ids are used */
  for (int s = 0; s < S; ++s)
    for (int j = 0; j < MAXNB; ++j) bt[s * MAXNB + j] = (j < (lens[s] + B - 1) / B) ? next-- : -1;
  const size_t pool_n = (size_t)P * Hkv * B * D;
  uint16_t* kp = malloc(pool_n * 2);
  uint16_t* vp = malloc(pool_n * 2);
  uint16_t* q = malloc((size_t)S * Hq * D * 2);
  uint16_t* kn = malloc((size_t)S * Hkv * D * 2);
  uint16_t* vn = malloc((size_t)S * Hkv * D * 2);
  for (size_t i = 0; i < pool_n; ++i) { kp[i] = rnd_bf16(); vp[i] = rnd_bf16(); }
  for (size_t i = 0; i < (size_t)S * Hq * D; ++i) q[i] = rnd_bf16();
  for (size_t i = 0; i < (size_t)S * Hkv * D; ++i) { kn[i] = rnd_bf16(); vn[i] = rnd_bf16(); }
  if (vox_oracle_kv_append(S, Hkv, D, B, P, MAXNB, kn, vn, kp, vp, bt, lens)) return 1;
  int64_t offs[S], total = 0;
  for (int s = 0; s < S; ++s) { offs[s] = total; total += lens[s]; }
  uint16_t* ko = malloc((size_t)total * Hkv * D * 2);
  uint16_t* vo = malloc((size_t)total * Hkv * D * 2);
  if (vox_oracle_kv_gather(S, Hkv, D, B, P, MAXNB, kp, vp, bt, lens, offs, ko, vo)) return 2;
  /* the gathered last row of every active stream is the appended row */
  for (int s = 0; s < S; ++s)
    if (lens[s] > 0)
      for (int i = 0; i < Hkv * D; ++i)
        if (ko[(offs[s] + lens[s] - 1) * Hkv * D + i] != kn[(size_t)s * Hkv * D + i]) return 3;
  double* out = malloc((size_t)S * Hq * D * sizeof(double));
  double* lse = malloc((size_t)S * Hq * sizeof(double));
  if (vox_oracle_paged_decode(S, Hq, Hkv, D, B, P, MAXNB, 0.125f, q, kp, vp, bt, lens, 0, S, out,
                              lse))
    return 4;
  for (int i = 0; i < S * Hq * D; ++i)
    if (!isfinite(out[i]) || fabs(out[i]) > 2.0) return 5; /* convex combination of |v| <= 2 */
  for (int i = 0; i < Hq; ++i)
    if (!(isinf(lse[3 * Hq + i]) && lse[3 * Hq + i] < 0)) return 6; /* stream 3 is inactive */
  /* subset call writes only its own rows */
  if (vox_oracle_paged_decode(S, Hq, Hkv, D, B, P, MAXNB, 0.125f, q, kp, vp, bt, lens, 4, 1, out,
                              NULL))
    return 7;
  /* multi-token step: whole prompts, a chunk, one token, nothing */
  const int32_t qo[S + 1] = {0, 1, 17, 20, 20, 31};
  enum { TQ = 31 };
  uint16_t* qm = malloc((size_t)TQ * Hq * D * 2);
  uint16_t* km = malloc((size_t)TQ * Hkv * D * 2);
  uint16_t* vm = malloc((size_t)TQ * Hkv * D * 2);
  for (size_t i = 0; i < (size_t)TQ * Hq * D; ++i) qm[i] = rnd_bf16();
  for (size_t i = 0; i < (size_t)TQ * Hkv * D; ++i) { km[i] = rnd_bf16(); vm[i] = rnd_bf16(); }
  if (vox_oracle_kv_append_multi(S, Hkv, D, B, P, MAXNB, km, vm, kp, vp, bt, lens, qo)) return 8;
  double* outm = malloc((size_t)TQ * Hq * D * sizeof(double));
  double* lsem = malloc((size_t)TQ * Hq * sizeof(double));
  if (vox_oracle_paged_prefill(S, Hq, Hkv, D, B, P, MAXNB, 0.125f, qm, kp, vp, bt, lens, qo, outm,
                               lsem))
    return 9;
  for (int i = 0; i < TQ * Hq * D; ++i)
    if (!isfinite(outm[i]) || fabs(outm[i]) > 2.0) return 10;
  /* rotary embedding + split + append; the table covers exactly the positions in use */
  enum { POS = 96 };
  float* rc = malloc((size_t)POS * (D / 2) * sizeof(float));
  float* rs = malloc((size_t)POS * (D / 2) * sizeof(float));
  for (int p = 0; p < POS; ++p)
    for (int i = 0; i < D / 2; ++i) {
      rc[p * (D / 2) + i] = cosf((float)p * 0.01f * (float)(i + 1));
      rs[p * (D / 2) + i] = sinf((float)p * 0.01f * (float)(i + 1));
    }
  uint16_t* qkv = malloc((size_t)S * (Hq + 2 * Hkv) * D * 2);
  uint16_t* qr = malloc((size_t)S * Hq * D * 2);
  for (size_t i = 0; i < (size_t)S * (Hq + 2 * Hkv) * D; ++i) qkv[i] = rnd_bf16();
  if (vox_oracle_rope_append(S, Hq, Hkv, D, B, P, MAXNB, qkv, rc, rs, POS, qr, kp, vp, bt, lens))
    return 11;
  if (vox_oracle_rope_append(S, Hq, Hkv, D, B, P, MAXNB, qkv, rc, rs, POS - 1, qr, kp, vp, bt,
                             lens) == 0)
    return 12; /* position 95 is outside a 95-row table */
  /* sampling: every mode, windows with empty and out-of-range slots */
  enum { SV = 301, SS = 6, SW = 5 };
  float* logits = malloc((size_t)SS * SV * sizeof(float));
  for (int i = 0; i < SS * SV; ++i) {
    state = state * 1664525u + 1013904223u;
    logits[i] = (float)((int)(state >> 16) % 2000 - 1000) / 100.0f;
  }
  const sampling_t prm[SS] = {{1.0f, 1.0f, 1.0f, 0},  {0.8f, 0.95f, 1.1f, 50}, {0.6f, 0.8f, 1.3f, 0},
                              {0.0f, 1.0f, 1.05f, 0}, {0.7f, 1e-9f, 1.0f, 3},  {1.0f, 1.0f, 1.0f, SV + 5}};
  const int32_t hist[SS * SW] = {-1, -1, -1, -1, -1, 0,  300, 5,  5,  -1, 7,   7, 7, 301, 9,
                                 12, 13, 14, 15, 16, -7, 1,   2,  3,  4,  300, 0, 1, 2,   3};
  const float us[SS] = {0.0f, 0.5f, 0.999999f, 0.3f, 0.9f, 0.25f};
  int32_t tok[SS], kept[SS];
  if (vox_oracle_sample(SS, SV, logits, prm, hist, SW, us, tok, kept)) return 13;
  for (int s = 0; s < SS; ++s)
    if (tok[s] < 0 || tok[s] >= SV || kept[s] < 1 || kept[s] > SV) return 14;
  if (kept[1] > 50 || kept[3] != 1 || kept[4] != 1 || kept[5] != SV) return 15;
  if (vox_oracle_sample(SS, SV, logits, prm, NULL, 0, us, tok, NULL)) return 16;
  free(logits);
  free(qm); free(km); free(vm); free(outm); free(lsem); free(rc); free(rs); free(qkv); free(qr);
  free(kp); free(vp); free(q); free(kn); free(vn); free(ko); free(vo); free(out); free(lse);
  puts("oracle sanitizer driver ok");
  return 0;
}
