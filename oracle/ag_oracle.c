/*
 * CPU oracle for the Attention-Gate (AG) inference path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the path computes, written from
 * the paper's definitions: the gate (Eq. 3 and Eq. 4, with the optional constant inside the
 * sigmoid from Sec. 3.5 "Initialization"), flag-masked causal attention (Eq. 2 under the
 * mask of Eq. 5), the KV-cache that retains only flagged tokens (Sec. 3.3, text after
 * Eq. 4), and one decoding step over that cache (Sec. 3.1, decoding stage).
 *
 * Storage is fp32 (bf16 inputs are widened by the caller); every reduction accumulates in
 * fp64 and results are returned in fp64.  Nothing is blocked, fused or reordered: the
 * attention loops run over the ORIGINAL, uncompacted keys with an `if` on the mask.
 * The only parallelism is one OpenMP loop over independent (batch, head) units.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use this file.  It
 * shares no code with the HIP library.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ag_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void ag_oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Gate threshold in logit space: Sigmoid(s) > tau  <=>  s > ln(tau / (1 - tau))  (Eq. 4;
 * the sigmoid is strictly increasing).  tau must lie in (0, 1). */
double ag_oracle_logit_threshold(double tau) { return log(tau / (1.0 - tau)); }

/*
 * Gate, Eq. 3 / Eq. 4 in the form "features -> h logits -> flags".
 *   feat  [B, L, d_in]   token features (hidden states for the linear variant of Sec. 3.4,
 *                        or the concatenated MHA' head outputs for the main architecture)
 *   w     [d_in, H_f]    projection to one logit per head (W^{O'} of Sec. 3.3)
 *   bias  [H_f]          constant added inside the sigmoid (gamma of Sec. 3.5, per head)
 *   logits[B, L, H_f]    s + bias in fp64
 *   flags [B, H_f, L]    1 = retain, 0 = evict; strict '>' so a tie evicts
 * The first n_sink tokens are forced to 1.  The comparison is made on the logit rounded to
 * fp32 against the threshold rounded to fp32, the precision the GPU path decides in.
 */
void ag_oracle_gate(const float *feat, const float *w, const float *bias, int B, int L, int d_in,
                    int H_f, double tau, int n_sink, double *logits, uint8_t *flags) {
  const float thr = (float)ag_oracle_logit_threshold(tau);
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b) {
    for (int t = 0; t < L; ++t) {
      const float *x = feat + ((size_t)b * L + t) * d_in;
      for (int h = 0; h < H_f; ++h) {
        double s = 0.0;
        for (int c = 0; c < d_in; ++c) s += (double)x[c] * (double)w[(size_t)c * H_f + h];
        s += (double)bias[h];
        logits[((size_t)b * L + t) * H_f + h] = s;
        uint8_t f = ((float)s > thr) ? 1 : 0;
        if (t < n_sink) f = 1;
        flags[((size_t)b * H_f + h) * L + t] = f;
      }
    }
  }
}

/* Eq. 5: is key column t visible to query row j under keep-flags f (of this head)?
 * n_recent = 1 is the paper's main setting (only the diagonal is always kept); a larger
 * value also keeps the n_recent-1 keys just before the query (Table 6 in the appendix "More Ablation", settings 6-1/6-2). */
static inline int visible(const uint8_t *f, int j, int t, int n_recent) {
  if (t > j) return 0;            /* j < t : causal               */
  if (j - t < n_recent) return 1; /* j = t (and the recent band)  */
  return f[t] != 0;               /* otherwise AG(X)^(t)          */
}

/*
 * One output row of Eq. 2 under the mask of Eq. 5: query row j of one head against the
 * keys/values 0..j of its KV head.  Q, K, V point at the head's [L, D] blocks, f at the
 * head's flags, z is scratch for L scores, o receives D values.  Masked columns contribute
 * exactly zero (the "large constant INF" of Eq. 2 taken as infinity).
 */
static void attn_row(const float *Q, const float *K, const float *V, const uint8_t *f, int j, int D,
                     double scale, int n_recent, double *z, double *o) {
  double m = -INFINITY;
  for (int t = 0; t <= j; ++t) {
    if (!visible(f, j, t, n_recent)) continue;
    double s = 0.0;
    for (int c = 0; c < D; ++c) s += (double)Q[(size_t)j * D + c] * (double)K[(size_t)t * D + c];
    z[t] = s * scale;
    if (z[t] > m) m = z[t];
  }
  double denom = 0.0;
  for (int c = 0; c < D; ++c) o[c] = 0.0;
  for (int t = 0; t <= j; ++t) {
    if (!visible(f, j, t, n_recent)) continue;
    const double p = exp(z[t] - m);
    denom += p;
    for (int c = 0; c < D; ++c) o[c] += p * (double)V[(size_t)t * D + c];
  }
  for (int c = 0; c < D; ++c) o[c] /= denom;
}

/*
 * Flag-masked causal attention, Eq. 2 with the mask of Eq. 5, one head at a time.
 *   q [B, Hq, L, D], k/v [B, Hkv, L, D], flags [B, Hkv, L], out [B, Hq, L, D] (fp64)
 * Query head i uses KV head i / (Hq / Hkv).
 */
void ag_oracle_prefill_attn(const float *q, const float *k, const float *v, const uint8_t *flags,
                            int B, int L, int Hq, int Hkv, int D, double scale, int n_recent,
                            double *out) {
  const int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < Hq; ++i) {
      const int g = i / G;
      const float *Q = q + ((size_t)b * Hq + i) * L * D;
      const float *K = k + ((size_t)b * Hkv + g) * L * D;
      const float *V = v + ((size_t)b * Hkv + g) * L * D;
      const uint8_t *f = flags + ((size_t)b * Hkv + g) * L;
      double *O = out + ((size_t)b * Hq + i) * L * D;
      double *z = (double *)malloc(sizeof(double) * (size_t)L);
      for (int j = 0; j < L; ++j) attn_row(Q, K, V, f, j, D, scale, n_recent, z, O + (size_t)j * D);
      free(z);
    }
  }
}

/*
 * The same rows, but only the query positions rows[0..n_rows) of every head (for checking
 * samples of a problem too large to compute whole).  out [B, Hq, n_rows, D] (fp64).
 */
void ag_oracle_prefill_rows(const float *q, const float *k, const float *v, const uint8_t *flags,
                            int B, int L, int Hq, int Hkv, int D, double scale, int n_recent,
                            const int32_t *rows, int n_rows, double *out) {
  const int G = Hq / Hkv;
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < Hq; ++i) {
      for (int r = 0; r < n_rows; ++r) {
        const int g = i / G;
        const float *Q = q + ((size_t)b * Hq + i) * L * D;
        const float *K = k + ((size_t)b * Hkv + g) * L * D;
        const float *V = v + ((size_t)b * Hkv + g) * L * D;
        const uint8_t *f = flags + ((size_t)b * Hkv + g) * L;
        double *z = (double *)malloc(sizeof(double) * (size_t)L);
        attn_row(Q, K, V, f, rows[r], D, scale, n_recent, z, out + (((size_t)b * Hq + i) * n_rows + r) * D);
        free(z);
      }
    }
  }
}

/*
 * KV-cache after prefilling: for each (batch, KV head) unit keep the rows whose flag is 1,
 * in increasing token order (Sec. 3.3: k, v of a token are retained iff AG = 1).
 *   k, v       [B*Hkv, L, row_bytes]  raw rows in the storage dtype (copied byte for byte)
 *   row_off    [B*Hkv + 1]            first cache row of each unit
 *   kc, vc     [total_rows, row_bytes]
 *   idx        [total_rows]           pos0 + original position of each cached row
 *   len        [B*Hkv]                rows kept
 * Returns the number of units whose kept rows exceed their capacity (those rows dropped).
 */
int ag_oracle_compact_kv(const uint8_t *k, const uint8_t *v, const uint8_t *flags, int n_units,
                         int L, size_t row_bytes, int pos0, const int64_t *row_off, uint8_t *kc,
                         uint8_t *vc, int32_t *idx, int32_t *len) {
  int overflow = 0;
  for (int u = 0; u < n_units; ++u) {
    const int64_t cap = row_off[u + 1] - row_off[u];
    int64_t c = 0;
    int over = 0;
    for (int t = 0; t < L; ++t) {
      if (!flags[(size_t)u * L + t]) continue;
      if (c >= cap) { over = 1; continue; }
      const size_t src = ((size_t)u * L + t) * row_bytes;
      const size_t dst = (size_t)(row_off[u] + c) * row_bytes;
      memcpy(kc + dst, k + src, row_bytes);
      memcpy(vc + dst, v + src, row_bytes);
      idx[row_off[u] + c] = pos0 + t;
      ++c;
    }
    len[u] = (int32_t)c;
    overflow += over;
  }
  return overflow;
}

/*
 * One decoding step (Sec. 3.1, decoding stage; the current token always attends to itself,
 * Eq. 5 diagonal).  For every (batch, query head): keys = cached rows ++ [k_new], same for
 * values, softmax-weighted sum.  Afterwards, per (batch, KV head): if new_flags is NULL or
 * new_flags[b, g] != 0, append (k_new, v_new, pos) to the cache.  All query heads of a group
 * read the cache before the append.
 *   q [B, Hq, D]; k_new, v_new [B, Hkv, D]; kc, vc [total_rows, D] fp32; out [B, Hq, D] fp64
 * Returns the number of units whose append was dropped for lack of capacity.
 */
int ag_oracle_decode_step(const float *q, const float *k_new, const float *v_new,
                          const uint8_t *new_flags, int pos, int B, int Hq, int Hkv, int D,
                          double scale, float *kc, float *vc, int32_t *idx, const int64_t *row_off,
                          int32_t *len, double *out) {
  const int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < Hq; ++i) {
      const int g = i / G;
      const int u = b * Hkv + g;
      const int n = len[u];
      const float *Q = q + ((size_t)b * Hq + i) * D;
      const float *K = kc + (size_t)row_off[u] * D;
      const float *V = vc + (size_t)row_off[u] * D;
      const float *kn = k_new + (size_t)u * D;
      const float *vn = v_new + (size_t)u * D;
      double *O = out + ((size_t)b * Hq + i) * D;
      double *z = (double *)malloc(sizeof(double) * (size_t)(n + 1));
      double m = -INFINITY;
      for (int t = 0; t <= n; ++t) {
        const float *kr = (t < n) ? K + (size_t)t * D : kn;
        double s = 0.0;
        for (int c = 0; c < D; ++c) s += (double)Q[c] * (double)kr[c];
        z[t] = s * scale;
        if (z[t] > m) m = z[t];
      }
      double denom = 0.0;
      for (int c = 0; c < D; ++c) O[c] = 0.0;
      for (int t = 0; t <= n; ++t) {
        const float *vr = (t < n) ? V + (size_t)t * D : vn;
        const double p = exp(z[t] - m);
        denom += p;
        for (int c = 0; c < D; ++c) O[c] += p * (double)vr[c];
      }
      for (int c = 0; c < D; ++c) O[c] /= denom;
      free(z);
    }
  }
  int dropped = 0;
  for (int u = 0; u < B * Hkv; ++u) {
    if (new_flags && !new_flags[u]) continue;
    const int64_t cap = row_off[u + 1] - row_off[u];
    if (len[u] >= cap) { ++dropped; continue; }
    const size_t r = (size_t)(row_off[u] + len[u]);
    memcpy(kc + r * D, k_new + (size_t)u * D, sizeof(float) * (size_t)D);
    memcpy(vc + r * D, v_new + (size_t)u * D, sizeof(float) * (size_t)D);
    idx[r] = pos;
    len[u] += 1;
  }
  return dropped;
}
