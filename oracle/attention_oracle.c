/*
 * fp64 CPU oracle for exact softmax attention and its analytic gradients.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU kernels are checked against.  It shares no code with them, and nothing on
 * the product path may call it.
 *
 * What is computed (per batch b, query head h, kv head g = h / (Hq/Hkv)).
 * The method (Sec. 2.1 "Transformer Architecture", Sec. 2.4 "SP-2", Sec. 4.2
 * "Computation Profiler": self-atten(b, S, H, D/s_sp) on one GPU) is the exact
 * multi-head softmax attention of the Transformer; the fused kernel the paper
 * names reaches exactly this result, so the oracle is the definition itself:
 *
 *   visible set V(i): tokens j of the same document as i, with j <= i when causal
 *   s_ij   = scale * sum_d q[i,h,d] * k[j,g,d]                 j in V(i)
 *   m_i    = max_j s_ij ;  l_i = sum_j exp(s_ij - m_i) ;  LSE_i = m_i + ln l_i
 *   p_ij   = exp(s_ij - LSE_i)
 *   o[i,h,:]  = sum_j p_ij * v[j,g,:]
 *   -- given dO --
 *   Delta_i   = sum_d dO[i,h,d] * o[i,h,d]
 *   dp_ij     = sum_d dO[i,h,d] * v[j,g,d]
 *   ds_ij     = p_ij * (dp_ij - Delta_i)
 *   dq[i,h,:] = scale * sum_j ds_ij * k[j,g,:]
 *   dk[j,g,:] = scale * sum_{h in group g} sum_{i : j in V(i)} ds_ij * q[i,h,:]
 *   dv[j,g,:] =         sum_{h in group g} sum_{i : j in V(i)} p_ij  * dO[i,h,:]
 *
 * Masked pairs are never formed (no -inf arithmetic).  Every row sees at least
 * itself, so no row is empty.  A document is a half-open token range
 * [cu[t], cu[t+1]); without cu the whole sequence of a batch entry is one document.
 *
 * Layouts (all fp64, contiguous): q, o, dout, dq: [B, S, Hq, D];  k, v, dk, dv:
 * [B, S, Hkv, D];  lse: [B, Hq, S].
 *
 * Three passes, each writing disjoint outputs so the summation order is fixed:
 *   pass 1 (rows)    -> lse, o
 *   pass 2 (rows)    -> dq
 *   pass 3 (columns) -> dk, dv      (recomputes s, p, dp)
 * Each pass takes a half-open token range and touches only those rows/columns,
 * which is how tests sample single rows of very long sequences.
 *
 * Parity pins (tests/test_oracle_pins.py): constant-V rows give exactly V; zero
 * queries give the running mean of V and LSE = ln(count); first row of a document
 * returns v of that token; block-diagonal packing equals per-document runs;
 * huge-margin scores give a one-hot; central finite differences for dq, dk, dv;
 * row sums of ds vanish; comparison with a library softmax/matmul/autograd.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_OK = 0, ORA_BAD_ARG = -1, ORA_NO_MEM = -2 };

typedef struct {
  int64_t B, S;
  int32_t Hq, Hkv, D, causal;
  double scale;
  int64_t *doc_begin; /* per token: first token of its document */
  int64_t *doc_end;   /* per token: one past the last token of its document */
} ora_shape;

static double dot(const double *a, const double *b, int32_t n) {
  double acc = 0.0;
#pragma omp simd reduction(+ : acc)
  for (int32_t d = 0; d < n; ++d) acc += a[d] * b[d];
  return acc;
}

static void axpy(double alpha, const double *x, double *y, int32_t n) {
#pragma omp simd
  for (int32_t d = 0; d < n; ++d) y[d] += alpha * x[d];
}

static int check_args(int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, const int32_t *cu, int32_t num_docs) {
  if (B < 1 || S < 1 || Hq < 1 || Hkv < 1 || D < 1) return ORA_BAD_ARG;
  if (Hq % Hkv != 0) return ORA_BAD_ARG;
  if (cu) {
    if (B != 1 || num_docs < 1) return ORA_BAD_ARG;
    if (cu[0] != 0 || cu[num_docs] != S) return ORA_BAD_ARG;
    for (int32_t t = 0; t < num_docs; ++t)
      if (cu[t + 1] < cu[t]) return ORA_BAD_ARG;
  }
  return ORA_OK;
}

/* Document bounds of every token. */
static int make_docs(ora_shape *sh, const int32_t *cu, int32_t num_docs) {
  sh->doc_begin = (int64_t *)malloc(sizeof(int64_t) * (size_t)sh->S);
  sh->doc_end = (int64_t *)malloc(sizeof(int64_t) * (size_t)sh->S);
  if (!sh->doc_begin || !sh->doc_end) return ORA_NO_MEM;
  if (!cu) {
    for (int64_t i = 0; i < sh->S; ++i) { sh->doc_begin[i] = 0; sh->doc_end[i] = sh->S; }
  } else {
    for (int32_t t = 0; t < num_docs; ++t)
      for (int64_t i = cu[t]; i < cu[t + 1]; ++i) { sh->doc_begin[i] = cu[t]; sh->doc_end[i] = cu[t + 1]; }
  }
  return ORA_OK;
}

static void free_docs(ora_shape *sh) { free(sh->doc_begin); free(sh->doc_end); }

/* First and one-past-last visible key of query token i. */
static void visible(const ora_shape *sh, int64_t i, int64_t *j0, int64_t *j1) {
  *j0 = sh->doc_begin[i];
  *j1 = sh->causal ? i + 1 : sh->doc_end[i];
}

/* Pass 1: lse and o for tokens row_begin <= i < row_end of every batch entry and head. */
int ora_attn_fwd(const double *q, const double *k, const double *v, double *o, double *lse,
                 const int32_t *cu_seqlens, int32_t num_docs, int64_t B, int64_t S, int32_t Hq, int32_t Hkv,
                 int32_t D, double scale, int32_t causal, int64_t row_begin, int64_t row_end) {
  int rc = check_args(B, S, Hq, Hkv, D, cu_seqlens, num_docs);
  if (rc) return rc;
  if (!q || !k || !v || !o || !lse || row_begin < 0 || row_end > S) return ORA_BAD_ARG;
  ora_shape sh = {B, S, Hq, Hkv, D, causal, scale, NULL, NULL};
  if ((rc = make_docs(&sh, cu_seqlens, num_docs))) { free_docs(&sh); return rc; }
  const int32_t group = Hq / Hkv;
  const int64_t nrows = row_end > row_begin ? row_end - row_begin : 0;
  int failed = 0;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * (size_t)S);
    if (!s) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for collapse(3) schedule(dynamic, 16)
      for (int64_t b = 0; b < B; ++b)
        for (int32_t h = 0; h < Hq; ++h)
          for (int64_t r = 0; r < nrows; ++r) {
            const int64_t i = row_begin + r;
            const int32_t g = h / group;
            const double *qi = q + ((b * S + i) * Hq + h) * D;
            int64_t j0, j1;
            visible(&sh, i, &j0, &j1);
            double m = -INFINITY;
            for (int64_t j = j0; j < j1; ++j) {
              s[j] = scale * dot(qi, k + ((b * S + j) * Hkv + g) * D, D);
              if (s[j] > m) m = s[j];
            }
            double l = 0.0;
            for (int64_t j = j0; j < j1; ++j) l += exp(s[j] - m);
            const double L = m + log(l);
            double *oi = o + ((b * S + i) * Hq + h) * D;
            for (int32_t d = 0; d < D; ++d) oi[d] = 0.0;
            for (int64_t j = j0; j < j1; ++j) axpy(exp(s[j] - L), v + ((b * S + j) * Hkv + g) * D, oi, D);
            lse[(b * Hq + h) * S + i] = L;
          }
    }
    free(s);
  }
  free_docs(&sh);
  return failed ? ORA_NO_MEM : ORA_OK;
}

/* Pass 2: dq for tokens row_begin <= i < row_end.  o and lse must hold pass 1's results for those rows. */
int ora_attn_bwd_dq(const double *q, const double *k, const double *v, const double *o, const double *dout,
                    const double *lse, double *dq, const int32_t *cu_seqlens, int32_t num_docs, int64_t B,
                    int64_t S, int32_t Hq, int32_t Hkv, int32_t D, double scale, int32_t causal,
                    int64_t row_begin, int64_t row_end) {
  int rc = check_args(B, S, Hq, Hkv, D, cu_seqlens, num_docs);
  if (rc) return rc;
  if (!q || !k || !v || !o || !dout || !lse || !dq || row_begin < 0 || row_end > S) return ORA_BAD_ARG;
  ora_shape sh = {B, S, Hq, Hkv, D, causal, scale, NULL, NULL};
  if ((rc = make_docs(&sh, cu_seqlens, num_docs))) { free_docs(&sh); return rc; }
  const int32_t group = Hq / Hkv;
  const int64_t nrows = row_end > row_begin ? row_end - row_begin : 0;
#pragma omp parallel for collapse(3) schedule(dynamic, 16)
  for (int64_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < Hq; ++h)
      for (int64_t r = 0; r < nrows; ++r) {
        const int64_t i = row_begin + r;
        const int32_t g = h / group;
        const int64_t qoff = ((b * S + i) * Hq + h) * D;
        const double *qi = q + qoff, *doi = dout + qoff;
        const double L = lse[(b * Hq + h) * S + i];
        const double delta = dot(doi, o + qoff, D);
        double *dqi = dq + qoff;
        for (int32_t d = 0; d < D; ++d) dqi[d] = 0.0;
        int64_t j0, j1;
        visible(&sh, i, &j0, &j1);
        for (int64_t j = j0; j < j1; ++j) {
          const double *kj = k + ((b * S + j) * Hkv + g) * D;
          const double *vj = v + ((b * S + j) * Hkv + g) * D;
          const double p = exp(scale * dot(qi, kj, D) - L);
          const double ds = p * (dot(doi, vj, D) - delta);
          axpy(ds, kj, dqi, D);
        }
        for (int32_t d = 0; d < D; ++d) dqi[d] *= scale;
      }
  free_docs(&sh);
  return ORA_OK;
}

/* Pass 3: dk and dv for key tokens col_begin <= j < col_end.  o and lse must hold pass 1's results for
 * every row that sees one of those keys (all later rows of the same documents when causal, the whole
 * documents otherwise). */
int ora_attn_bwd_dkdv(const double *q, const double *k, const double *v, const double *o, const double *dout,
                      const double *lse, double *dk, double *dv, const int32_t *cu_seqlens, int32_t num_docs,
                      int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, double scale, int32_t causal,
                      int64_t col_begin, int64_t col_end) {
  int rc = check_args(B, S, Hq, Hkv, D, cu_seqlens, num_docs);
  if (rc) return rc;
  if (!q || !k || !v || !o || !dout || !lse || !dk || !dv || col_begin < 0 || col_end > S) return ORA_BAD_ARG;
  ora_shape sh = {B, S, Hq, Hkv, D, causal, scale, NULL, NULL};
  if ((rc = make_docs(&sh, cu_seqlens, num_docs))) { free_docs(&sh); return rc; }
  const int32_t group = Hq / Hkv;
  const int64_t ncols = col_end > col_begin ? col_end - col_begin : 0;
#pragma omp parallel for collapse(3) schedule(dynamic, 16)
  for (int64_t b = 0; b < B; ++b)
    for (int32_t g = 0; g < Hkv; ++g)
      for (int64_t c = 0; c < ncols; ++c) {
        const int64_t j = col_begin + c;
        const int64_t koff = ((b * S + j) * Hkv + g) * D;
        const double *kj = k + koff, *vj = v + koff;
        double *dkj = dk + koff, *dvj = dv + koff;
        for (int32_t d = 0; d < D; ++d) { dkj[d] = 0.0; dvj[d] = 0.0; }
        /* rows that see key j: same document, and i >= j when causal */
        const int64_t i0 = causal ? j : sh.doc_begin[j];
        const int64_t i1 = sh.doc_end[j];
        for (int32_t h = g * group; h < (g + 1) * group; ++h)
          for (int64_t i = i0; i < i1; ++i) {
            const int64_t qoff = ((b * S + i) * Hq + h) * D;
            const double *qi = q + qoff, *doi = dout + qoff;
            const double delta = dot(doi, o + qoff, D);
            const double p = exp(scale * dot(qi, kj, D) - lse[(b * Hq + h) * S + i]);
            const double ds = p * (dot(doi, vj, D) - delta);
            axpy(ds, qi, dkj, D);
            axpy(p, doi, dvj, D);
          }
        for (int32_t d = 0; d < D; ++d) dkj[d] *= scale;
      }
  free_docs(&sh);
  return ORA_OK;
}

int ora_num_threads(void) {
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
