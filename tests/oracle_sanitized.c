/* The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only; compiled together with
 * oracle/ag_oracle.c by tests/test_oracle_pins.py).  Every buffer is heap-allocated at exactly the size the
 * oracle's contract states, so a read or write one element past an array, an overflowing index or a misaligned
 * access aborts the run.  Shapes are chosen at the edges: L = 1, a prompt shorter than the recent window, GQA, an
 * empty and a full unit, a cache with no room and one with exactly enough. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double ag_oracle_logit_threshold(double tau);
void ag_oracle_gate(const float *feat, const float *w, const float *bias, int B, int L, int d_in, int H_f, double tau,
                    int n_sink, double *logits, uint8_t *flags);
void ag_oracle_prefill_attn(const float *q, const float *k, const float *v, const uint8_t *flags, int B, int L, int Hq,
                            int Hkv, int D, double scale, int n_recent, double *out);
void ag_oracle_prefill_rows(const float *q, const float *k, const float *v, const uint8_t *flags, int B, int L, int Hq,
                            int Hkv, int D, double scale, int n_recent, const int32_t *rows, int n_rows, double *out);
int ag_oracle_compact_kv(const uint8_t *k, const uint8_t *v, const uint8_t *flags, int n_units, int L, size_t row_bytes,
                         int pos0, const int64_t *row_off, uint8_t *kc, uint8_t *vc, int32_t *idx, int32_t *len);
int ag_oracle_decode_step(const float *q, const float *k_new, const float *v_new, const uint8_t *new_flags, int pos, int B,
                          int Hq, int Hkv, int D, double scale, float *kc, float *vc, int32_t *idx,
                          const int64_t *row_off, int32_t *len, double *out);

static uint32_t state = 12345u;
static float rnd(void) {
  state = state * 1664525u + 1013904223u;
  return (float)((state >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static float *fvec(size_t n) {
  float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) p[i] = rnd();
  return p;
}

static int finite_all(const double *x, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!isfinite(x[i])) return 0;
  return 1;
}

static int one_case(int B, int L, int Hq, int Hkv, int D, int d_in, int n_recent, int cap_slack) {
  const int U = B * Hkv;
  float *x = fvec((size_t)B * L * d_in), *w = fvec((size_t)d_in * Hkv), *bias = fvec((size_t)Hkv);
  double *logits = (double *)malloc(sizeof(double) * (size_t)B * L * Hkv);
  uint8_t *flags = (uint8_t *)malloc((size_t)U * L);
  ag_oracle_gate(x, w, bias, B, L, d_in, Hkv, 0.5, 1, logits, flags);
  if (U > 1) memset(flags + (size_t)(U - 1) * L, 0, (size_t)L);          /* one fully evicted unit */
  memset(flags, 1, (size_t)L);                                           /* one unit that keeps everything */
  float *q = fvec((size_t)B * Hq * L * D), *k = fvec((size_t)U * L * D), *v = fvec((size_t)U * L * D);
  double *out = (double *)malloc(sizeof(double) * (size_t)B * Hq * L * D);
  ag_oracle_prefill_attn(q, k, v, flags, B, L, Hq, Hkv, D, 0.25, n_recent, out);
  if (!finite_all(out, (size_t)B * Hq * L * D)) return 1;
  int32_t rows[3] = {0, L - 1, L / 2};
  double *some = (double *)malloc(sizeof(double) * (size_t)B * Hq * 3 * D);
  ag_oracle_prefill_rows(q, k, v, flags, B, L, Hq, Hkv, D, 0.25, n_recent, rows, 3, some);
  for (int d = 0; d < D; ++d)
    if (some[(size_t)1 * D + d] != out[(size_t)(L - 1) * D + d]) return 2;   /* head 0, row L - 1 */
  /* compaction into slabs of L + cap_slack rows (cap_slack < 0: too small, rows dropped) */
  const int cap = L + cap_slack > 0 ? L + cap_slack : 0;
  int64_t *ro = (int64_t *)malloc(sizeof(int64_t) * (size_t)(U + 1));
  for (int u = 0; u <= U; ++u) ro[u] = (int64_t)u * cap;
  const size_t total = (size_t)U * cap;
  float *kc = (float *)malloc(sizeof(float) * (total ? total : 1) * D), *vc = (float *)malloc(sizeof(float) * (total ? total : 1) * D);
  int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (total ? total : 1)), *len = (int32_t *)malloc(sizeof(int32_t) * (size_t)U);
  const int over = ag_oracle_compact_kv((const uint8_t *)k, (const uint8_t *)v, flags, U, L, sizeof(float) * (size_t)D, 7,
                                        ro, (uint8_t *)kc, (uint8_t *)vc, idx, len);
  if (cap_slack >= 0 && over != 0) return 3;
  if (cap_slack < 0 && over == 0) return 4;                              /* unit 0 keeps L rows: must overflow */
  for (int u = 0; u < U; ++u)
    if (len[u] < 0 || len[u] > cap) return 5;
  /* decode: cap_slack steps fit exactly in unit 0, one more is dropped */
  float *dq = fvec((size_t)B * Hq * D), *kn = fvec((size_t)U * D), *vn = fvec((size_t)U * D);
  double *o = (double *)malloc(sizeof(double) * (size_t)B * Hq * D);
  const int steps = (cap_slack > 0 ? cap_slack : 0) + 1;
  for (int s = 0; s < steps; ++s) {
    const int dropped = ag_oracle_decode_step(dq, kn, vn, NULL, L + s, B, Hq, Hkv, D, 0.25, kc, vc, idx, ro, len, o);
    if (!finite_all(o, (size_t)B * Hq * D)) return 6;
    if (s + 1 < steps && cap_slack > 0 && len[0] != L + s + 1) return 7;
    if (s + 1 == steps && dropped < 1) return 8;                         /* unit 0 is full by now */
  }
  free(x); free(w); free(bias); free(logits); free(flags); free(q); free(k); free(v); free(out); free(some); free(ro);
  free(kc); free(vc); free(idx); free(len); free(dq); free(kn); free(vn); free(o);
  return 0;
}

int main(void) {
  if (fabs(ag_oracle_logit_threshold(0.5)) > 1e-15) return 100;
  const int cases[][8] = {
      /* B, L, Hq, Hkv, D, d_in, n_recent, cap_slack */
      {1, 1, 1, 1, 4, 8, 1, 0},   {1, 1, 2, 1, 4, 8, 5, 2},  {2, 7, 4, 2, 8, 16, 1, 3}, {1, 33, 8, 2, 16, 32, 10, 1},
      {2, 65, 3, 3, 4, 8, 64, 0}, {1, 40, 4, 4, 8, 8, 3, -5}, {3, 5, 2, 2, 4, 4, 8, -5},
  };
  for (unsigned c = 0; c < sizeof(cases) / sizeof(cases[0]); ++c) {
    const int *a = cases[c];
    const int rc = one_case(a[0], a[1], a[2], a[3], a[4], a[5], a[6], a[7]);
    if (rc) { printf("case %u failed with %d\n", c, rc); return (int)(10 * (c + 1) + rc); }
  }
  puts("ok");
  return 0;
}
