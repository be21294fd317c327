/*
 * moda_ref.c -- fp64 CPU oracle for Mixture-of-Depths Attention (MoDA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * definition that the HIP kernels are checked against.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the GPU path and links no HIP.
 *
 * What it computes (paper section 2.2 "Mixture-of-Depths Attention", Eq. 2 for
 * the sequence part, Algorithm 1 for the index sets and the single shared
 * normaliser):
 *
 *   for every batch b, query head h (kv head g = h / G, G = Hq / Hk) and
 *   position t, ONE softmax runs over the union of
 *     - the sequence keys  Kseq[b,g,j]      j <= t  (j < T if not causal;
 *       Eq. 2's mask is 0 for j <= i, so the diagonal is visible), and
 *     - the depth keys     Kdepth[b,g,t,i]  i < depth_count, all taken at
 *       the query's own position t (section 2.2 "Depth Attention": a token
 *       attends only to the depth keys/values of the same token position;
 *       Algorithm 1's depth mask floor(i_q/G) == floor(j_d/L)),
 *   with logits scale * <q, k> (Eq. 2's 1/sqrt(d)), and the output is the
 *   weighted sum of the matching values divided by the one normaliser
 *   (Algorithm 1: o <- o / acc).  LSE = max + ln(normaliser) in natural-log
 *   units; the paper's base-2 online update is an evaluation order for the
 *   same base-e softmax, so this file uses exp()/log().
 *
 * The implementation literally builds the concatenated (logit, value pointer)
 * list for a query and runs a two-pass naive softmax over it.  No tiling, no
 * online update, no fusion.
 *
 * The backward pass is not given by the paper; it is the derivative of the
 * definition above, written as closed forms (see moda_ref_bwd_f64).
 *
 * Layouts (row-major, contiguous, double precision, host pointers):
 *   Q, O, dO, dQ           [B, Hq, T, d]
 *   Kseq, Vseq, grads      [B, Hk, T, d]
 *   Kdepth, Vdepth, grads  [B, Hk, T, depth_alloc, d]  (slots < depth_count used)
 *   LSE                    [B, Hq, T]
 * Return value: 0 on success, 1 on a bad argument.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int B, Hq, Hk, T, d, depth_alloc, depth_count, causal;
  double scale;
} ref_shape;

static int shape_ok(const ref_shape* s) {
  if (s->B < 0 || s->Hq <= 0 || s->Hk <= 0 || s->T < 0 || s->d <= 0) return 0;
  if (s->Hq % s->Hk != 0) return 0;
  if (s->depth_count < 0 || s->depth_alloc < s->depth_count) return 0;
  if (!(s->scale > 0.0)) return 0;
  return 1;
}

static double dot(const double* a, const double* b, int d) {
  double s = 0.0;
  for (int k = 0; k < d; ++k) s += a[k] * b[k];
  return s;
}

/* Number of threads the parallel loops will use (for reporting). */
int moda_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * One query.  kseq/vseq point at the [T, d] slab of the query's kv head,
 * kdep/vdep at the [depth_alloc, d] slab of position t (may be NULL when
 * depth_count == 0).  n_seq = number of visible sequence keys (t+1 or T).
 * Builds the explicit concatenation: entries [0, n_seq) are sequence keys,
 * entries [n_seq, n_seq + depth_count) are the depth slots.
 * Writes o[d], *lse and, if w != NULL, the n_seq + depth_count weights.
 */
static void one_query(const double* q, const double* kseq, const double* vseq, int n_seq,
                      const double* kdep, const double* vdep, int depth_count, int d,
                      double scale, double* logit, const double** val, double* o, double* lse,
                      double* w) {
  int n = 0;
  for (int j = 0; j < n_seq; ++j) {
    logit[n] = scale * dot(q, kseq + (size_t)j * d, d);
    val[n] = vseq + (size_t)j * d;
    ++n;
  }
  for (int i = 0; i < depth_count; ++i) {
    logit[n] = scale * dot(q, kdep + (size_t)i * d, d);
    val[n] = vdep + (size_t)i * d;
    ++n;
  }
  /* pass 1: maximum over the union; pass 2: one normaliser over the union */
  double m = -INFINITY;
  for (int c = 0; c < n; ++c)
    if (logit[c] > m) m = logit[c];
  double z = 0.0;
  for (int c = 0; c < n; ++c) z += exp(logit[c] - m);
  for (int k = 0; k < d; ++k) o[k] = 0.0;
  for (int c = 0; c < n; ++c) {
    double p = exp(logit[c] - m) / z;
    if (w) w[c] = p;
    for (int k = 0; k < d; ++k) o[k] += p * val[c][k];
  }
  *lse = m + log(z);
}

/*
 * Forward for a list of query positions rows[0..n_rows) (each in [0,T)), for
 * all b and h.  Q_rows is [B,Hq,n_rows,d]; Kdepth_rows/Vdepth_rows are
 * [B,Hk,n_rows,depth_alloc,d] (the depth slabs of those positions only, so a
 * long-context sample does not need the whole depth tensor on the host);
 * Kseq/Vseq are the full [B,Hk,T,d].  Outputs O_rows [B,Hq,n_rows,d],
 * LSE_rows [B,Hq,n_rows].
 */
int moda_ref_fwd_rows_f64(const double* Q_rows, const double* Kseq, const double* Vseq,
                          const double* Kdepth_rows, const double* Vdepth_rows,
                          const int* rows, int n_rows, double* O_rows, double* LSE_rows,
                          int B, int Hq, int Hk, int T, int d, int depth_alloc,
                          int depth_count, int causal, double scale) {
  ref_shape s = {B, Hq, Hk, T, d, depth_alloc, depth_count, causal, scale};
  if (!shape_ok(&s) || n_rows < 0) return 1;
  if (!Q_rows || !Kseq || !Vseq || !O_rows || !LSE_rows || (n_rows > 0 && !rows)) return 1;
  if (depth_count > 0 && (!Kdepth_rows || !Vdepth_rows)) return 1;
  for (int r = 0; r < n_rows; ++r)
    if (rows[r] < 0 || rows[r] >= T) return 1;
  const int G = Hq / Hk;
  const long long total = (long long)B * Hq * n_rows;
  int fail = 0;
#pragma omp parallel
  {
    double* logit = (double*)malloc(sizeof(double) * (size_t)(T + depth_count + 1));
    const double** val = (const double**)malloc(sizeof(double*) * (size_t)(T + depth_count + 1));
    if (!logit || !val) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 4)
      for (long long idx = 0; idx < total; ++idx) {
        int r = (int)(idx % n_rows);
        int h = (int)((idx / n_rows) % Hq);
        int b = (int)(idx / ((long long)n_rows * Hq));
        int g = h / G;
        int t = rows[r];
        const double* q = Q_rows + ((size_t)(b * Hq + h) * n_rows + r) * d;
        const double* ks = Kseq + (size_t)(b * Hk + g) * T * d;
        const double* vs = Vseq + (size_t)(b * Hk + g) * T * d;
        const double* kd = NULL;
        const double* vd = NULL;
        if (depth_count > 0) {
          size_t off = ((size_t)(b * Hk + g) * n_rows + r) * (size_t)depth_alloc * d;
          kd = Kdepth_rows + off;
          vd = Vdepth_rows + off;
        }
        int n_seq = causal ? t + 1 : T;
        one_query(q, ks, vs, n_seq, kd, vd, depth_count, d, scale, logit, val,
                  O_rows + ((size_t)(b * Hq + h) * n_rows + r) * d,
                  LSE_rows + (size_t)(b * Hq + h) * n_rows + r, NULL);
      }
    }
    free(logit);
    free((void*)val);
  }
  return fail;
}

/* Forward for every position: the rows variant with rows = 0..T-1. */
int moda_ref_fwd_f64(const double* Q, const double* Kseq, const double* Vseq,
                     const double* Kdepth, const double* Vdepth, double* O, double* LSE,
                     int B, int Hq, int Hk, int T, int d, int depth_alloc, int depth_count,
                     int causal, double scale) {
  if (T < 0) return 1;
  if (T == 0 || B == 0) return 0;
  int* rows = (int*)malloc(sizeof(int) * (size_t)T);
  if (!rows) return 1;
  for (int t = 0; t < T; ++t) rows[t] = t;
  int rc = moda_ref_fwd_rows_f64(Q, Kseq, Vseq, Kdepth, Vdepth, rows, T, O, LSE, B, Hq, Hk, T, d,
                                 depth_alloc, depth_count, causal, scale);
  free(rows);
  return rc;
}

/*
 * Debug entry: the softmax weights of one query (b,h,t) over the explicit
 * union.  w must hold n_seq + depth_count doubles (sequence keys first, in
 * order, then the depth slots); n_seq = t+1 if causal else T.
 */
int moda_ref_weights_f64(const double* Q, const double* Kseq, const double* Vseq,
                         const double* Kdepth, const double* Vdepth, int b, int h, int t,
                         double* w, int B, int Hq, int Hk, int T, int d, int depth_alloc,
                         int depth_count, int causal, double scale) {
  ref_shape s = {B, Hq, Hk, T, d, depth_alloc, depth_count, causal, scale};
  if (!shape_ok(&s) || b < 0 || b >= B || h < 0 || h >= Hq || t < 0 || t >= T || !w) return 1;
  if (depth_count > 0 && (!Kdepth || !Vdepth)) return 1;
  int g = h / (Hq / Hk);
  int n_seq = causal ? t + 1 : T;
  double* logit = (double*)malloc(sizeof(double) * (size_t)(n_seq + depth_count + 1));
  const double** val = (const double**)malloc(sizeof(double*) * (size_t)(n_seq + depth_count + 1));
  double* o = (double*)malloc(sizeof(double) * (size_t)d);
  if (!logit || !val || !o) return 1;
  double lse;
  size_t doff = ((size_t)(b * Hk + g) * T + t) * (size_t)depth_alloc * d;
  one_query(Q + ((size_t)(b * Hq + h) * T + t) * d, Kseq + (size_t)(b * Hk + g) * T * d,
            Vseq + (size_t)(b * Hk + g) * T * d, n_seq, depth_count ? Kdepth + doff : NULL,
            depth_count ? Vdepth + doff : NULL, depth_count, d, scale, logit, val, o, &lse, w);
  free(logit);
  free((void*)val);
  free(o);
  return 0;
}

/*
 * Backward.  The paper states no backward algorithm; these are the
 * derivatives of the forward definition above.  For a query (b,h,t) with
 * softmax weights p_c over the union (c runs over its sequence keys and its
 * depth slots), output o = sum_c p_c v_c, upstream gradient g = dO[b,h,t] and
 * delta = <g, o>:
 *     dv_c += p_c * g
 *     e_c   = p_c * (<g, v_c> - delta)            (gradient w.r.t. logit c)
 *     dq   += scale * e_c * k_c
 *     dk_c += scale * e_c * q
 * A sequence key c = j accumulates over every query that sees it (and over
 * the G query heads of its kv head); a depth slot (t,i) is seen only by the
 * queries at position t (G of them under GQA).
 * Everything, including o, is recomputed here in fp64 from the inputs.
 *
 * Parallelised over (b, kv head) so that no two threads touch the same
 * gradient element.  Any of the five gradient pointers may be NULL to skip it
 * (dKdepth/dVdepth must be NULL or valid when depth_count == 0; they are then
 * untouched).  Depth gradient slots >= depth_count are written as zero.
 */
int moda_ref_bwd_f64(const double* Q, const double* Kseq, const double* Vseq,
                     const double* Kdepth, const double* Vdepth, const double* dO, double* dQ,
                     double* dKseq, double* dVseq, double* dKdepth, double* dVdepth, int B,
                     int Hq, int Hk, int T, int d, int depth_alloc, int depth_count, int causal,
                     double scale) {
  ref_shape s = {B, Hq, Hk, T, d, depth_alloc, depth_count, causal, scale};
  if (!shape_ok(&s)) return 1;
  if (!Q || !Kseq || !Vseq || !dO) return 1;
  if (depth_count > 0 && (!Kdepth || !Vdepth)) return 1;
  const int G = Hq / Hk;
  int fail = 0;
#pragma omp parallel
  {
    size_t nmax = (size_t)T + depth_count + 1;
    double* logit = (double*)malloc(sizeof(double) * nmax);
    const double** val = (const double**)malloc(sizeof(double*) * nmax);
    double* w = (double*)malloc(sizeof(double) * nmax);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    if (!logit || !val || !w || !o) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int bg = 0; bg < B * Hk; ++bg) {
        int b = bg / Hk, g = bg % Hk;
        const double* ks = Kseq + (size_t)bg * T * d;
        const double* vs = Vseq + (size_t)bg * T * d;
        double* dks = dKseq ? dKseq + (size_t)bg * T * d : NULL;
        double* dvs = dVseq ? dVseq + (size_t)bg * T * d : NULL;
        if (dks) memset(dks, 0, sizeof(double) * (size_t)T * d);
        if (dvs) memset(dvs, 0, sizeof(double) * (size_t)T * d);
        if (depth_alloc > 0) {
          size_t nd = (size_t)T * depth_alloc * d;
          if (dKdepth) memset(dKdepth + (size_t)bg * nd, 0, sizeof(double) * nd);
          if (dVdepth) memset(dVdepth + (size_t)bg * nd, 0, sizeof(double) * nd);
        }
        for (int hh = 0; hh < G; ++hh) {
          int h = g * G + hh;
          for (int t = 0; t < T; ++t) {
            size_t qoff = ((size_t)(b * Hq + h) * T + t) * d;
            const double* q = Q + qoff;
            const double* go = dO + qoff;
            size_t doff = ((size_t)bg * T + t) * (size_t)depth_alloc * d;
            const double* kd = depth_count ? Kdepth + doff : NULL;
            const double* vd = depth_count ? Vdepth + doff : NULL;
            int n_seq = causal ? t + 1 : T;
            double lse;
            one_query(q, ks, vs, n_seq, kd, vd, depth_count, d, scale, logit, val, o, &lse, w);
            double delta = dot(go, o, d);
            double* dq = dQ ? dQ + qoff : NULL;
            if (dq)
              for (int k = 0; k < d; ++k) dq[k] = 0.0;
            for (int c = 0; c < n_seq + depth_count; ++c) {
              const double* kc;
              double *dkc, *dvc;
              if (c < n_seq) {
                kc = ks + (size_t)c * d;
                dkc = dks ? dks + (size_t)c * d : NULL;
                dvc = dvs ? dvs + (size_t)c * d : NULL;
              } else {
                size_t so = doff + (size_t)(c - n_seq) * d;
                kc = Kdepth + so;
                dkc = dKdepth ? dKdepth + so : NULL;
                dvc = dVdepth ? dVdepth + so : NULL;
              }
              double e = w[c] * (dot(go, val[c], d) - delta);
              for (int k = 0; k < d; ++k) {
                if (dvc) dvc[k] += w[c] * go[k];
                if (dq) dq[k] += scale * e * kc[k];
                if (dkc) dkc[k] += scale * e * q[k];
              }
            }
          }
        }
      }
    }
    free(logit);
    free((void*)val);
    free(w);
    free(o);
  }
  return fail;
}

/*
 * Rounding-noise scale of the backward (an analysis helper for the parity
 * tests' tolerance; the paper gives neither a backward algorithm nor an error
 * figure for it, Table 2 only times it).
 *
 * Model: an implementation of the formulas of moda_ref_bwd_f64 that
 *   (a) rounds every softmax weight p_c and every logit gradient e_c, each
 *       (query, key) pair independently, with a relative error of standard
 *       deviation u before the products that sum over queries or keys, and
 *   (b) receives an output o of the forward whose elements carry independent
 *       relative errors of standard deviation u (the forward's output
 *       rounding), so that delta = <g, o> is off by a random amount of
 *       standard deviation u * D_t, D_t = sqrt(sum_k (g_k o_k)^2), the same
 *       amount for every key of the query (e_c is then off by -p_c times it).
 * To first order in u the error of each gradient element is a sum of
 * independent terms; this function returns its standard deviation for u = 1:
 *     nV_c[k]^2 = sum_t (p_tc g_t[k])^2
 *     nK_c[k]^2 = scale^2 sum_t ((e_tc q_t[k])^2 + (p_tc D_t q_t[k])^2)
 *     nQ_t[k]^2 = scale^2 (sum_c (e_tc k_c[k])^2 + (D_t sum_c p_tc k_c[k])^2)
 * (sums over t run over the queries, and the G query heads, that see key c).
 * Arguments and layouts as in moda_ref_bwd_f64; any output may be NULL.
 */
int moda_ref_bwd_noise_f64(const double* Q, const double* Kseq, const double* Vseq,
                           const double* Kdepth, const double* Vdepth, const double* dO, double* nQ,
                           double* nKseq, double* nVseq, double* nKdepth, double* nVdepth, int B,
                           int Hq, int Hk, int T, int d, int depth_alloc, int depth_count, int causal,
                           double scale) {
  ref_shape s = {B, Hq, Hk, T, d, depth_alloc, depth_count, causal, scale};
  if (!shape_ok(&s)) return 1;
  if (!Q || !Kseq || !Vseq || !dO) return 1;
  if (depth_count > 0 && (!Kdepth || !Vdepth)) return 1;
  const int G = Hq / Hk;
  int fail = 0;
#pragma omp parallel
  {
    size_t nmax = (size_t)T + depth_count + 1;
    double* logit = (double*)malloc(sizeof(double) * nmax);
    const double** val = (const double**)malloc(sizeof(double*) * nmax);
    double* w = (double*)malloc(sizeof(double) * nmax);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    double* kbar = (double*)malloc(sizeof(double) * (size_t)d);
    if (!logit || !val || !w || !o || !kbar) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int bg = 0; bg < B * Hk; ++bg) {
        int b = bg / Hk, g = bg % Hk;
        const double* ks = Kseq + (size_t)bg * T * d;
        const double* vs = Vseq + (size_t)bg * T * d;
        double* nks = nKseq ? nKseq + (size_t)bg * T * d : NULL;
        double* nvs = nVseq ? nVseq + (size_t)bg * T * d : NULL;
        size_t nd = (size_t)T * depth_alloc * d;
        double* nkd = (nKdepth && depth_alloc > 0) ? nKdepth + (size_t)bg * nd : NULL;
        double* nvd = (nVdepth && depth_alloc > 0) ? nVdepth + (size_t)bg * nd : NULL;
        /* the variances are summed in place; the square root is taken at the end */
        if (nks) memset(nks, 0, sizeof(double) * (size_t)T * d);
        if (nvs) memset(nvs, 0, sizeof(double) * (size_t)T * d);
        if (nkd) memset(nkd, 0, sizeof(double) * nd);
        if (nvd) memset(nvd, 0, sizeof(double) * nd);
        for (int hh = 0; hh < G; ++hh) {
          int h = g * G + hh;
          for (int t = 0; t < T; ++t) {
            size_t qoff = ((size_t)(b * Hq + h) * T + t) * d;
            const double* q = Q + qoff;
            const double* go = dO + qoff;
            size_t doff_local = (size_t)t * depth_alloc * d;
            const double* kd = depth_count ? Kdepth + (size_t)bg * nd + doff_local : NULL;
            const double* vd = depth_count ? Vdepth + (size_t)bg * nd + doff_local : NULL;
            int n_seq = causal ? t + 1 : T;
            double lse;
            one_query(q, ks, vs, n_seq, kd, vd, depth_count, d, scale, logit, val, o, &lse, w);
            double delta = dot(go, o, d);
            double D2 = 0.0;
            for (int k = 0; k < d; ++k) D2 += (go[k] * o[k]) * (go[k] * o[k]);
            for (int k = 0; k < d; ++k) kbar[k] = 0.0;
            double* nq = nQ ? nQ + qoff : NULL;
            if (nq)
              for (int k = 0; k < d; ++k) nq[k] = 0.0;
            for (int c = 0; c < n_seq + depth_count; ++c) {
              const double* kc;
              double *nkc, *nvc;
              if (c < n_seq) {
                kc = ks + (size_t)c * d;
                nkc = nks ? nks + (size_t)c * d : NULL;
                nvc = nvs ? nvs + (size_t)c * d : NULL;
              } else {
                size_t so = doff_local + (size_t)(c - n_seq) * d;
                kc = kd + (size_t)(c - n_seq) * d;
                nkc = nkd ? nkd + so : NULL;
                nvc = nvd ? nvd + so : NULL;
              }
              double e = w[c] * (dot(go, val[c], d) - delta);
              for (int k = 0; k < d; ++k) {
                kbar[k] += w[c] * kc[k];
                if (nvc) nvc[k] += (w[c] * go[k]) * (w[c] * go[k]);
                if (nq) nq[k] += (scale * e * kc[k]) * (scale * e * kc[k]);
                if (nkc) nkc[k] += (scale * q[k]) * (scale * q[k]) * (e * e + w[c] * w[c] * D2);
              }
            }
            if (nq)
              for (int k = 0; k < d; ++k)
                nq[k] = sqrt(nq[k] + (scale * kbar[k]) * (scale * kbar[k]) * D2);
          }
        }
        if (nks) for (size_t i = 0; i < (size_t)T * d; ++i) nks[i] = sqrt(nks[i]);
        if (nvs) for (size_t i = 0; i < (size_t)T * d; ++i) nvs[i] = sqrt(nvs[i]);
        if (nkd) for (size_t i = 0; i < nd; ++i) nkd[i] = sqrt(nkd[i]);
        if (nvd) for (size_t i = 0; i < nd; ++i) nvd[i] = sqrt(nvd[i]);
      }
    }
    free(logit);
    free((void*)val);
    free(w);
    free(o);
    free(kbar);
  }
  return fail;
}

/*
 * Backward, row-local gradients only, for a list of positions rows[0..n_rows):
 * dQ_rows [B,Hq,n_rows,d] and dKdepth_rows/dVdepth_rows
 * [B,Hk,n_rows,depth_alloc,d] (either may be NULL).  These depend only on the
 * query's own row, so a long problem can be checked on a sample.  Inputs as in
 * moda_ref_fwd_rows_f64 plus dO_rows [B,Hq,n_rows,d].  Same formulas as
 * moda_ref_bwd_f64.
 */
int moda_ref_bwd_rows_f64(const double* Q_rows, const double* Kseq, const double* Vseq,
                          const double* Kdepth_rows, const double* Vdepth_rows,
                          const double* dO_rows, const int* rows, int n_rows, double* dQ_rows,
                          double* dKdepth_rows, double* dVdepth_rows, int B, int Hq, int Hk,
                          int T, int d, int depth_alloc, int depth_count, int causal,
                          double scale) {
  ref_shape s = {B, Hq, Hk, T, d, depth_alloc, depth_count, causal, scale};
  if (!shape_ok(&s) || n_rows < 0) return 1;
  if (!Q_rows || !Kseq || !Vseq || !dO_rows || (n_rows > 0 && !rows)) return 1;
  if (depth_count > 0 && (!Kdepth_rows || !Vdepth_rows)) return 1;
  for (int r = 0; r < n_rows; ++r)
    if (rows[r] < 0 || rows[r] >= T) return 1;
  const int G = Hq / Hk;
  int fail = 0;
#pragma omp parallel
  {
    size_t nmax = (size_t)T + depth_count + 1;
    double* logit = (double*)malloc(sizeof(double) * nmax);
    const double** val = (const double**)malloc(sizeof(double*) * nmax);
    double* w = (double*)malloc(sizeof(double) * nmax);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    if (!logit || !val || !w || !o) {
#pragma omp atomic write
      fail = 1;
    } else {
      /* one (b, kv head, row) per iteration: the G heads of the group are
         looped inside so that the depth gradients have a single writer */
#pragma omp for schedule(dynamic, 4)
      for (long long idx = 0; idx < (long long)B * Hk * n_rows; ++idx) {
        int r = (int)(idx % n_rows);
        int bg = (int)(idx / n_rows);
        int b = bg / Hk, g = bg % Hk;
        int t = rows[r];
        const double* ks = Kseq + (size_t)bg * T * d;
        const double* vs = Vseq + (size_t)bg * T * d;
        size_t doff = ((size_t)bg * n_rows + r) * (size_t)depth_alloc * d;
        const double* kd = depth_count ? Kdepth_rows + doff : NULL;
        const double* vd = depth_count ? Vdepth_rows + doff : NULL;
        if (depth_alloc > 0) {
          if (dKdepth_rows) memset(dKdepth_rows + doff, 0, sizeof(double) * (size_t)depth_alloc * d);
          if (dVdepth_rows) memset(dVdepth_rows + doff, 0, sizeof(double) * (size_t)depth_alloc * d);
        }
        int n_seq = causal ? t + 1 : T;
        for (int hh = 0; hh < G; ++hh) {
          int h = g * G + hh;
          size_t qoff = ((size_t)(b * Hq + h) * n_rows + r) * d;
          const double* q = Q_rows + qoff;
          const double* go = dO_rows + qoff;
          double lse;
          one_query(q, ks, vs, n_seq, kd, vd, depth_count, d, scale, logit, val, o, &lse, w);
          double delta = dot(go, o, d);
          double* dq = dQ_rows ? dQ_rows + qoff : NULL;
          if (dq)
            for (int k = 0; k < d; ++k) dq[k] = 0.0;
          for (int c = 0; c < n_seq + depth_count; ++c) {
            double e = w[c] * (dot(go, val[c], d) - delta);
            const double* kc = c < n_seq ? ks + (size_t)c * d : kd + (size_t)(c - n_seq) * d;
            if (dq)
              for (int k = 0; k < d; ++k) dq[k] += scale * e * kc[k];
            if (c >= n_seq) {
              size_t so = doff + (size_t)(c - n_seq) * d;
              for (int k = 0; k < d; ++k) {
                if (dKdepth_rows) dKdepth_rows[so + k] += scale * e * q[k];
                if (dVdepth_rows) dVdepth_rows[so + k] += w[c] * go[k];
              }
            }
          }
        }
      }
    }
    free(logit);
    free((void*)val);
    free(w);
    free(o);
  }
  return fail;
}

/*
 * Rounding-noise scale (see moda_ref_bwd_noise_f64) of the row-local
 * gradients for a list of positions; arguments and layouts as in
 * moda_ref_bwd_rows_f64.
 */
int moda_ref_bwd_noise_rows_f64(const double* Q_rows, const double* Kseq, const double* Vseq,
                                const double* Kdepth_rows, const double* Vdepth_rows,
                                const double* dO_rows, const int* rows, int n_rows, double* nQ_rows,
                                double* nKdepth_rows, double* nVdepth_rows, int B, int Hq, int Hk,
                                int T, int d, int depth_alloc, int depth_count, int causal,
                                double scale) {
  ref_shape s = {B, Hq, Hk, T, d, depth_alloc, depth_count, causal, scale};
  if (!shape_ok(&s) || n_rows < 0) return 1;
  if (!Q_rows || !Kseq || !Vseq || !dO_rows || (n_rows > 0 && !rows)) return 1;
  if (depth_count > 0 && (!Kdepth_rows || !Vdepth_rows)) return 1;
  for (int r = 0; r < n_rows; ++r)
    if (rows[r] < 0 || rows[r] >= T) return 1;
  const int G = Hq / Hk;
  int fail = 0;
#pragma omp parallel
  {
    size_t nmax = (size_t)T + depth_count + 1;
    double* logit = (double*)malloc(sizeof(double) * nmax);
    const double** val = (const double**)malloc(sizeof(double*) * nmax);
    double* w = (double*)malloc(sizeof(double) * nmax);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    double* kbar = (double*)malloc(sizeof(double) * (size_t)d);
    if (!logit || !val || !w || !o || !kbar) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 4)
      for (long long idx = 0; idx < (long long)B * Hk * n_rows; ++idx) {
        int r = (int)(idx % n_rows);
        int bg = (int)(idx / n_rows);
        int b = bg / Hk, g = bg % Hk;
        int t = rows[r];
        const double* ks = Kseq + (size_t)bg * T * d;
        const double* vs = Vseq + (size_t)bg * T * d;
        size_t doff = ((size_t)bg * n_rows + r) * (size_t)depth_alloc * d;
        const double* kd = depth_count ? Kdepth_rows + doff : NULL;
        const double* vd = depth_count ? Vdepth_rows + doff : NULL;
        size_t nslot = (size_t)depth_alloc * d;
        if (depth_alloc > 0) {
          if (nKdepth_rows) memset(nKdepth_rows + doff, 0, sizeof(double) * nslot);
          if (nVdepth_rows) memset(nVdepth_rows + doff, 0, sizeof(double) * nslot);
        }
        int n_seq = causal ? t + 1 : T;
        for (int hh = 0; hh < G; ++hh) {
          int h = g * G + hh;
          size_t qoff = ((size_t)(b * Hq + h) * n_rows + r) * d;
          const double* q = Q_rows + qoff;
          const double* go = dO_rows + qoff;
          double lse;
          one_query(q, ks, vs, n_seq, kd, vd, depth_count, d, scale, logit, val, o, &lse, w);
          double delta = dot(go, o, d);
          double D2 = 0.0;
          for (int k = 0; k < d; ++k) D2 += (go[k] * o[k]) * (go[k] * o[k]);
          for (int k = 0; k < d; ++k) kbar[k] = 0.0;
          double* nq = nQ_rows ? nQ_rows + qoff : NULL;
          if (nq)
            for (int k = 0; k < d; ++k) nq[k] = 0.0;
          for (int c = 0; c < n_seq + depth_count; ++c) {
            double e = w[c] * (dot(go, val[c], d) - delta);
            const double* kc = c < n_seq ? ks + (size_t)c * d : kd + (size_t)(c - n_seq) * d;
            for (int k = 0; k < d; ++k) {
              kbar[k] += w[c] * kc[k];
              if (nq) nq[k] += (scale * e * kc[k]) * (scale * e * kc[k]);
            }
            if (c >= n_seq) {
              size_t so = doff + (size_t)(c - n_seq) * d;
              for (int k = 0; k < d; ++k) {
                if (nKdepth_rows)
                  nKdepth_rows[so + k] += (scale * q[k]) * (scale * q[k]) * (e * e + w[c] * w[c] * D2);
                if (nVdepth_rows) nVdepth_rows[so + k] += (w[c] * go[k]) * (w[c] * go[k]);
              }
            }
          }
          if (nq)
            for (int k = 0; k < d; ++k) nq[k] = sqrt(nq[k] + (scale * kbar[k]) * (scale * kbar[k]) * D2);
        }
        if (depth_alloc > 0) {
          if (nKdepth_rows) for (size_t i = 0; i < nslot; ++i) nKdepth_rows[doff + i] = sqrt(nKdepth_rows[doff + i]);
          if (nVdepth_rows) for (size_t i = 0; i < nslot; ++i) nVdepth_rows[doff + i] = sqrt(nVdepth_rows[doff + i]);
        }
      }
    }
    free(logit);
    free((void*)val);
    free(w);
    free(o);
    free(kbar);
  }
  return fail;
}
