/*
 * fp64 CPU oracle for causal attention over one packed buffer.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may link, load or call this file;
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline leg have an
 * independent, slow, obviously correct statement of what the GPU kernels must compute.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it computes.  The paper (Section 1, third paragraph; Appendix D, layer cost
 * 24Bsh^2 + 4B*sum s_i^2; Algorithm 7, a = sum len(x)^2) states only that the attention of a
 * pack is the sum of the attentions of its samples: every token attends inside its own
 * sample.  The attention itself is the textbook scaled-dot-product softmax with a causal
 * mask, written out here as its definition, one query row (or one key column) at a time:
 *
 *   sample i owns packed rows cu[i] <= r < cu[i+1]; query head h reads kv head h / (Hq/Hkv)
 *   S[r,k]   = scale * sum_j Q[r,h,j] K[k,kh,j]            for cu[i] <= k <= r
 *   LSE[h,r] = m + ln sum_k exp(S[r,k] - m),  m = max_k S[r,k]
 *   P[r,k]   = exp(S[r,k] - LSE[h,r]);    O[r,h,:] = sum_k P[r,k] V[k,kh,:]
 *   backward of L = sum O.dO:   D[r] = sum_x dO[r,h,x] O[r,h,x]
 *   dP[r,k]  = sum_x dO[r,h,x] V[k,kh,x];   dS[r,k] = P[r,k] (dP[r,k] - D[r])
 *   dQ[r,h,:]  = scale * sum_k dS[r,k] K[k,kh,:]
 *   dK[k,kh,:] = scale * sum_{h in group kh} sum_{r>=k, same sample} dS[r,k] Q[r,h,:]
 *   dV[k,kh,:] =         sum_{h in group kh} sum_{r>=k, same sample} P[r,k] dO[r,h,:]
 *
 * Inputs are float32 arrays whose values are the bf16-rounded tensors (so the GPU path and
 * this file see identical numbers); every product and sum is carried in double.  There is no
 * tiling, no running-max softmax and no fusion: each row materialises its whole score vector.
 * Row and column subsets let the large packs be checked on sampled outputs.
 *
 * Layouts: Q [T,Hq,d], K [T,Hkv,d], V [T,Hkv,e], dO [T,Hq,e], all dense row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  const float *q, *k, *v, *d_o;
  const int32_t *cu;
  int n, T, Hq, Hkv, d, e;
  double scale;
} problem;

static int check_problem(const problem *p) {
  if (!p->q || !p->k || !p->v || !p->cu) return 1;
  if (p->n < 0 || p->T < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->d <= 0 || p->e <= 0) return 2;
  if (p->Hq % p->Hkv) return 3;
  if (p->cu[0] != 0) return 4;
  for (int i = 0; i < p->n; ++i)
    if (p->cu[i + 1] < p->cu[i]) return 4;
  if (p->cu[p->n] != p->T) return 4;
  return 0;
}

/* first packed row of the sample that owns row r */
static int sample_begin(const problem *p, int r) {
  for (int i = 0; i < p->n; ++i)
    if (r >= p->cu[i] && r < p->cu[i + 1]) return p->cu[i];
  return -1;
}
static int sample_end(const problem *p, int r) {
  for (int i = 0; i < p->n; ++i)
    if (r >= p->cu[i] && r < p->cu[i + 1]) return p->cu[i + 1];
  return -1;
}
static int max_sample_len(const problem *p) {
  int m = 1;
  for (int i = 0; i < p->n; ++i)
    if (p->cu[i + 1] - p->cu[i] > m) m = p->cu[i + 1] - p->cu[i];
  return m;
}

/* One query row r of head h: scores s[0..r-c], probabilities pr[0..r-c], output o[0..e), lse. */
static void row_forward(const problem *p, int h, int r, int c, double *s, double *pr, double *o,
                        double *lse_out) {
  const int kh = h / (p->Hq / p->Hkv);
  const float *qrow = p->q + ((size_t)r * p->Hq + h) * p->d;
  double m = -INFINITY;
  for (int k = c; k <= r; ++k) {
    const float *krow = p->k + ((size_t)k * p->Hkv + kh) * p->d;
    double acc = 0.0;
    for (int j = 0; j < p->d; ++j) acc += (double)qrow[j] * (double)krow[j];
    s[k - c] = p->scale * acc;
    if (s[k - c] > m) m = s[k - c];
  }
  double sum = 0.0;
  for (int k = c; k <= r; ++k) sum += exp(s[k - c] - m);
  const double lse = m + log(sum);
  for (int x = 0; x < p->e; ++x) o[x] = 0.0;
  for (int k = c; k <= r; ++k) {
    const float *vrow = p->v + ((size_t)k * p->Hkv + kh) * p->e;
    const double w = exp(s[k - c] - lse);
    pr[k - c] = w;
    for (int x = 0; x < p->e; ++x) o[x] += w * (double)vrow[x];
  }
  *lse_out = lse;
}

/*
 * Forward on a subset of rows (rows == NULL: all T rows, n_rows must be T).
 * O   [n_rows, Hq, e]  double
 * LSE [Hq, n_rows]     double
 */
int hbp_oracle_fwd(const float *q, const float *k, const float *v, const int32_t *cu, int n, int T,
                   int Hq, int Hkv, int d, int e, double scale, const int32_t *rows, int n_rows,
                   double *O, double *LSE) {
  problem p = {q, k, v, NULL, cu, n, T, Hq, Hkv, d, e, scale};
  int rc = check_problem(&p);
  if (rc) return rc;
  if (!O || !LSE || n_rows < 0) return 1;
  if (!rows && n_rows != T) return 5;
  for (int i = 0; i < n_rows; ++i) {
    int r = rows ? rows[i] : i;
    if (r < 0 || r >= T) return 5;
  }
  const int smax = max_sample_len(&p);
  const long total = (long)n_rows * Hq;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * smax);
    double *pr = (double *)malloc(sizeof(double) * smax);
#pragma omp for schedule(dynamic, 4)
    for (long it = 0; it < total; ++it) {
      const int i = (int)(it / Hq), h = (int)(it % Hq);
      const int r = rows ? rows[i] : i;
      const int c = sample_begin(&p, r);
      row_forward(&p, h, r, c, s, pr, O + ((size_t)i * Hq + h) * e, LSE + (size_t)h * n_rows + i);
    }
    free(s);
    free(pr);
  }
  return 0;
}

/*
 * dQ on a subset of rows (rows == NULL: all rows).  dQ [n_rows, Hq, d] double.
 * Optionally also returns D [Hq, n_rows] (may be NULL).
 */
int hbp_oracle_bwd_dq(const float *q, const float *k, const float *v, const float *d_o,
                      const int32_t *cu, int n, int T, int Hq, int Hkv, int d, int e, double scale,
                      const int32_t *rows, int n_rows, double *dQ, double *Dout) {
  problem p = {q, k, v, d_o, cu, n, T, Hq, Hkv, d, e, scale};
  int rc = check_problem(&p);
  if (rc) return rc;
  if (!d_o || !dQ || n_rows < 0) return 1;
  if (!rows && n_rows != T) return 5;
  for (int i = 0; i < n_rows; ++i) {
    int r = rows ? rows[i] : i;
    if (r < 0 || r >= T) return 5;
  }
  const int smax = max_sample_len(&p);
  const long total = (long)n_rows * Hq;
  const int g = Hq / Hkv;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * smax);
    double *pr = (double *)malloc(sizeof(double) * smax);
    double *o = (double *)malloc(sizeof(double) * e);
#pragma omp for schedule(dynamic, 4)
    for (long it = 0; it < total; ++it) {
      const int i = (int)(it / Hq), h = (int)(it % Hq);
      const int r = rows ? rows[i] : i;
      const int c = sample_begin(&p, r);
      const int kh = h / g;
      double lse;
      row_forward(&p, h, r, c, s, pr, o, &lse);
      const float *dorow = d_o + ((size_t)r * Hq + h) * e;
      double D = 0.0;
      for (int x = 0; x < e; ++x) D += (double)dorow[x] * o[x];
      if (Dout) Dout[(size_t)h * n_rows + i] = D;
      double *dq = dQ + ((size_t)i * Hq + h) * d;
      for (int j = 0; j < d; ++j) dq[j] = 0.0;
      for (int kk = c; kk <= r; ++kk) {
        const float *vrow = v + ((size_t)kk * Hkv + kh) * e;
        const float *krow = k + ((size_t)kk * Hkv + kh) * d;
        double dP = 0.0;
        for (int x = 0; x < e; ++x) dP += (double)dorow[x] * (double)vrow[x];
        const double dS = pr[kk - c] * (dP - D);
        for (int j = 0; j < d; ++j) dq[j] += dS * (double)krow[j];
      }
      for (int j = 0; j < d; ++j) dq[j] *= scale;
    }
    free(s);
    free(pr);
    free(o);
  }
  return 0;
}

/*
 * dK, dV on a subset of key columns (cols == NULL: all T).
 * dK [n_cols, Hkv, d], dV [n_cols, Hkv, e] double.
 * Needs LSE and D of every row r >= k of the same sample, which it computes itself first.
 */
int hbp_oracle_bwd_dkdv(const float *q, const float *k, const float *v, const float *d_o,
                        const int32_t *cu, int n, int T, int Hq, int Hkv, int d, int e,
                        double scale, const int32_t *cols, int n_cols, double *dK, double *dV) {
  problem p = {q, k, v, d_o, cu, n, T, Hq, Hkv, d, e, scale};
  int rc = check_problem(&p);
  if (rc) return rc;
  if (!d_o || !dK || !dV || n_cols < 0) return 1;
  if (!cols && n_cols != T) return 5;
  for (int i = 0; i < n_cols; ++i) {
    int c = cols ? cols[i] : i;
    if (c < 0 || c >= T) return 5;
  }
  const int g = Hq / Hkv;
  const int smax = max_sample_len(&p);

  /* rows whose LSE and D are needed: from the smallest selected column of each sample on */
  int32_t *first_needed = (int32_t *)malloc(sizeof(int32_t) * (n > 0 ? n : 1));
  for (int i = 0; i < n; ++i) first_needed[i] = cu[i + 1]; /* none */
  for (int i = 0; i < n_cols; ++i) {
    const int c = cols ? cols[i] : i;
    for (int sidx = 0; sidx < n; ++sidx)
      if (c >= cu[sidx] && c < cu[sidx + 1] && c < first_needed[sidx]) first_needed[sidx] = c;
  }
  double *lse = (double *)calloc((size_t)Hq * (T > 0 ? T : 1), sizeof(double));
  double *D = (double *)calloc((size_t)Hq * (T > 0 ? T : 1), sizeof(double));
  int32_t *need_rows = (int32_t *)malloc(sizeof(int32_t) * (T > 0 ? T : 1));
  int n_need = 0;
  for (int sidx = 0; sidx < n; ++sidx)
    for (int r = first_needed[sidx]; r < cu[sidx + 1]; ++r) need_rows[n_need++] = r;
  const long total_rows = (long)n_need * Hq;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * smax);
    double *pr = (double *)malloc(sizeof(double) * smax);
    double *o = (double *)malloc(sizeof(double) * e);
#pragma omp for schedule(dynamic, 4)
    for (long it = 0; it < total_rows; ++it) {
      const int r = need_rows[it / Hq], h = (int)(it % Hq);
      const int c = sample_begin(&p, r);
      double l;
      row_forward(&p, h, r, c, s, pr, o, &l);
      const float *dorow = d_o + ((size_t)r * Hq + h) * e;
      double acc = 0.0;
      for (int x = 0; x < e; ++x) acc += (double)dorow[x] * o[x];
      lse[(size_t)h * T + r] = l;
      D[(size_t)h * T + r] = acc;
    }
    free(s);
    free(pr);
    free(o);
  }

  const long total = (long)n_cols * Hkv;
#pragma omp parallel for schedule(dynamic, 1)
  for (long it = 0; it < total; ++it) {
    const int i = (int)(it / Hkv), kh = (int)(it % Hkv);
    const int kk = cols ? cols[i] : i;
    const int end = sample_end(&p, kk);
    const float *krow = k + ((size_t)kk * Hkv + kh) * d;
    const float *vrow = v + ((size_t)kk * Hkv + kh) * e;
    double *dk = dK + ((size_t)i * Hkv + kh) * d;
    double *dv = dV + ((size_t)i * Hkv + kh) * e;
    for (int j = 0; j < d; ++j) dk[j] = 0.0;
    for (int x = 0; x < e; ++x) dv[x] = 0.0;
    for (int h = kh * g; h < (kh + 1) * g; ++h) {
      for (int r = kk; r < end; ++r) {
        const float *qrow = q + ((size_t)r * Hq + h) * d;
        const float *dorow = d_o + ((size_t)r * Hq + h) * e;
        double sc = 0.0;
        for (int j = 0; j < d; ++j) sc += (double)qrow[j] * (double)krow[j];
        const double P = exp(scale * sc - lse[(size_t)h * T + r]);
        double dP = 0.0;
        for (int x = 0; x < e; ++x) dP += (double)dorow[x] * (double)vrow[x];
        const double dS = P * (dP - D[(size_t)h * T + r]);
        for (int x = 0; x < e; ++x) dv[x] += P * (double)dorow[x];
        for (int j = 0; j < d; ++j) dk[j] += dS * (double)qrow[j];
      }
    }
    for (int j = 0; j < d; ++j) dk[j] *= scale;
  }
  free(first_needed);
  free(lse);
  free(D);
  free(need_rows);
  return 0;
}

/* Probability row P[r, cu_i..r] of head h (for the rows-sum-to-one and sum dS = 0 pins). */
int hbp_oracle_prob_row(const float *q, const float *k, const float *v, const int32_t *cu, int n,
                        int T, int Hq, int Hkv, int d, int e, double scale, int h, int r,
                        double *P_out /* [r - c + 1] */, int *len_out) {
  problem p = {q, k, v, NULL, cu, n, T, Hq, Hkv, d, e, scale};
  int rc = check_problem(&p);
  if (rc) return rc;
  if (h < 0 || h >= Hq || r < 0 || r >= T || !P_out || !len_out) return 5;
  const int c = sample_begin(&p, r);
  double *s = (double *)malloc(sizeof(double) * (r - c + 1));
  double *o = (double *)malloc(sizeof(double) * e);
  double lse;
  row_forward(&p, h, r, c, s, P_out, o, &lse);
  *len_out = r - c + 1;
  free(s);
  free(o);
  return 0;
}

int hbp_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
