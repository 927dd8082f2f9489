/*
 * ReST-KV eviction path -- CPU ORACLE (test infrastructure, not the product).
 *
 * A plain, slow, double-precision implementation of what the eviction path
 * computes, written from the paper's definitions.  It exists so that the HIP
 * library can be checked against something that can be read against the paper
 * by eye.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it; it shares no code with the HIP path.
 *
 * Conventions (0-indexed):
 *   L   cached tokens, W observation-window queries (positions L-W .. L-1),
 *   P = L - W evictable prefix tokens, d head dimension, G query heads that
 *   share one KV head.  Inputs are float arrays whose values are exactly the
 *   ones the GPU receives (bf16 inputs are widened, not re-rounded); every
 *   intermediate and every output is double.
 *
 * Steps and the passages they follow:
 *   attention weights / outputs        Sec. 3.1, Eq. (softmax), Eq. (mha)
 *   leave-one-out indicator            Sec. 3.2, Eq. (ori); App. A Eq. (ori_2)
 *   closed-form indicator              Sec. 3.2, Eq. (rec_ei); App. A Eq. (relation)..(last_eq)
 *   EMA temporal smoothing             Sec. 3.3, EMA recursion
 *   adaptive-window spatial smoothing  Sec. 3.3, D_front/D_rear, W_s, gamma_shift, Eq. (final_ei)
 *   selection and gather               Sec. 3.3, Eq. (topk)
 *   ablation variants                  Sec. 4 (ablation table), App. on the ablation study:
 *                                      attention-weight and value-norm indicators, mean and
 *                                      inverse-EMA temporal smoothing, max pooling
 *
 * Readings of points the paper leaves open are listed where they are applied
 * and, together, in the design document of this repository.
 *
 * Parity unpinned (no independent check exists; both are design readings):
 *   - how the G query heads of one KV head are combined (mean of the per-head
 *     indicator, rk_oracle_group_mean);
 *   - how the fixed kernel size k of App. B combines with the W_s equation
 *     (rk_oracle_aws_window, k > 1);
 *   - the maximum over the group as the alternative GQA reduction (rk_oracle_group_max) and
 *     the meaning of "Inv-EMA" (rk_oracle_temporal, mode 2), which the paper names but does
 *     not define: the functions themselves are pinned to their stated definitions.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define RK_OK 0
#define RK_EINVAL (-1)
#define RK_ENOMEM (-2)

int rk_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Attention of one query over its visible keys: Eq. (softmax).               */
/* e[n] = exp(s[n]-max) for n < nvis, *l_out = sum e.  A[n] = e[n] / l.       */
/* If logit is not NULL it receives the scaled logits s[n].                    */
static void softmax_row(const float* q, const float* k, int d, int64_t nvis,
                        double scale, double* e, double* l_out, double* logit) {
  double mx = -INFINITY;
  for (int64_t n = 0; n < nvis; ++n) {
    double s = 0.0;
    const float* kn = k + n * (int64_t)d;
    for (int c = 0; c < d; ++c) s += (double)q[c] * (double)kn[c];
    s *= scale;
    e[n] = s;
    if (logit) logit[n] = s;
    if (s > mx) mx = s;
  }
  double l = 0.0;
  for (int64_t n = 0; n < nvis; ++n) {
    e[n] = exp(e[n] - mx);
    l += e[n];
  }
  *l_out = l;
}

/* number of keys query i of the window can see */
static int64_t visible(int64_t L, int64_t W, int64_t i, int causal) {
  return causal ? (L - W + i + 1) : L;
}

/*
 * Attention weights and head outputs of the window queries.
 * q [Hq,W,d], k,v [Hkv,L,d]; A [Hq,W,L] (zero where masked), z [Hq,W,d].
 * Query head h reads KV head h / (Hq/Hkv).  Either output may be NULL.
 */
int rk_oracle_attention(const float* q, const float* k, const float* v, int Hq,
                        int Hkv, int d, int64_t L, int64_t W, double scale,
                        int causal, double* A, double* z) {
  if (!q || !k || !v || Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || W < 1 || W > L)
    return RK_EINVAL;
  const int G = Hq / Hkv;
  int rc = RK_OK;
#pragma omp parallel for schedule(dynamic)
  for (int64_t hi = 0; hi < (int64_t)Hq * W; ++hi) {
    const int h = (int)(hi / W);
    const int64_t i = hi % W;
    const int g = h / G;
    const float* kg = k + (int64_t)g * L * d;
    const float* vg = v + (int64_t)g * L * d;
    const int64_t nvis = visible(L, W, i, causal);
    double* e = (double*)malloc(sizeof(double) * (size_t)L);
    if (!e) { rc = RK_ENOMEM; continue; }
    double l;
    softmax_row(q + hi * d, kg, d, nvis, scale, e, &l, NULL);
    if (A) {
      double* Arow = A + hi * L;
      for (int64_t n = 0; n < L; ++n) Arow[n] = n < nvis ? e[n] / l : 0.0;
    }
    if (z) {
      double* zr = z + hi * d;
      for (int c = 0; c < d; ++c) zr[c] = 0.0;
      for (int64_t n = 0; n < nvis; ++n) {
        const double a = e[n] / l;
        for (int c = 0; c < d; ++c) zr[c] += a * (double)vg[n * d + c];
      }
    }
    free(e);
  }
  return rc;
}

/* y[r] = sum_c x[c] * fac[c*r_dim + r]  (x W_O for one head; fac NULL = identity) */
static void project(const double* x, const double* fac, int d, int r_dim, double* y) {
  if (!fac) {
    for (int c = 0; c < d; ++c) y[c] = x[c];
    return;
  }
  for (int r = 0; r < r_dim; ++r) y[r] = 0.0;
  for (int c = 0; c < d; ++c) {
    const double xc = x[c];
    const double* fr = fac + (int64_t)c * r_dim;
    for (int r = 0; r < r_dim; ++r) y[r] += xc * fr[r];
  }
}

static double norm2(const double* a, const double* b, int n) {
  double s = 0.0;
  for (int i = 0; i < n; ++i) {
    const double t = a[i] - b[i];
    s += t * t;
  }
  return sqrt(s);
}

/*
 * Leave-one-out indicator, Eq. (ori), by brute force: for every prefix token n
 * the key/value pair is removed, the softmax over the remaining visible keys is
 * recomputed from the logits, and the l2 distance of the two projected head
 * outputs is taken.
 *
 * One KV head:  q [G,nq,d]; qpos[nq] = absolute position of each query (it
 * sees keys 0..qpos) or -1 to see all L keys; k,v [L,d]; fac [G,d,r_dim] is
 * the output projection of each query head (z W_O orientation; NULL = identity,
 * r_dim = d); I [G,nq,P].  O(P * L * d) per query: tiny inputs only.
 */
int rk_oracle_indicator_loo(const float* q, const int64_t* qpos, const float* k,
                            const float* v, const double* fac, int r_dim, int G,
                            int nq, int d, int64_t L, int64_t P, double scale,
                            double* I) {
  if (!q || !k || !v || !I || G <= 0 || nq <= 0 || d <= 0 || P < 0 || P > L) return RK_EINVAL;
  if (!fac) r_dim = d;
  int rc = RK_OK;
#pragma omp parallel for schedule(dynamic)
  for (int64_t hq = 0; hq < (int64_t)G * nq; ++hq) {
    const int h = (int)(hq / nq);
    const int64_t i = hq % nq;
    const int64_t nvis = (qpos && qpos[i] >= 0) ? qpos[i] + 1 : L;
    const double* fh = fac ? fac + (int64_t)h * d * r_dim : NULL;
    double* s = (double*)malloc(sizeof(double) * (size_t)L);
    double* zf = (double*)malloc(sizeof(double) * (size_t)d);
    double* zr = (double*)malloc(sizeof(double) * (size_t)d);
    double* yf = (double*)malloc(sizeof(double) * (size_t)r_dim);
    double* yr = (double*)malloc(sizeof(double) * (size_t)r_dim);
    if (!s || !zf || !zr || !yf || !yr) {
      rc = RK_ENOMEM;
    } else {
      const float* qr = q + hq * d;
      for (int64_t n = 0; n < nvis; ++n) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += (double)qr[c] * (double)k[n * d + c];
        s[n] = acc * scale;
      }
      /* full cache */
      {
        double mx = -INFINITY, l = 0.0;
        for (int64_t n = 0; n < nvis; ++n) if (s[n] > mx) mx = s[n];
        for (int c = 0; c < d; ++c) zf[c] = 0.0;
        for (int64_t n = 0; n < nvis; ++n) l += exp(s[n] - mx);
        for (int64_t n = 0; n < nvis; ++n) {
          const double a = exp(s[n] - mx) / l;
          for (int c = 0; c < d; ++c) zf[c] += a * (double)v[n * d + c];
        }
        project(zf, fh, d, r_dim, yf);
      }
      for (int64_t rm = 0; rm < P; ++rm) {
        double* out = I + hq * P + rm;
        if (rm >= nvis) { *out = 0.0; continue; }   /* an invisible key changes nothing */
        if (nvis == 1) { *out = 0.0; continue; }    /* nothing left to attend to */
        double mx = -INFINITY, l = 0.0;
        for (int64_t n = 0; n < nvis; ++n) if (n != rm && s[n] > mx) mx = s[n];
        for (int64_t n = 0; n < nvis; ++n) if (n != rm) l += exp(s[n] - mx);
        for (int c = 0; c < d; ++c) zr[c] = 0.0;
        for (int64_t n = 0; n < nvis; ++n) {
          if (n == rm) continue;
          const double a = exp(s[n] - mx) / l;
          for (int c = 0; c < d; ++c) zr[c] += a * (double)v[n * d + c];
        }
        project(zr, fh, d, r_dim, yr);
        *out = norm2(yf, yr, r_dim);
      }
    }
    free(s); free(zf); free(zr); free(yf); free(yr);
  }
  return rc;
}

/*
 * Closed-form indicator, Eq. (rec_ei):
 *     I[n] = A[n] / (1 - A[n]) * || z W_O - v_n W_O ||_2 .
 * Same argument layout as rk_oracle_indicator_loo.  The projection "fac" may
 * be the explicit per-head W_O [d, D] or any [d, r] factor F with
 * F F^T = W_O W_O^T (the norm only depends on that product).
 *
 * 1 - A[n] is formed as (l - e[n]) / l from the unnormalised weights.  A token
 * that holds more than half of the attention mass (there is at most one per
 * query) makes the closed form a quotient of two vanishing quantities; for it
 * the definition Eq. (ori) is evaluated instead -- App. A shows the two are the
 * same number -- with the remaining weights renormalised by Eq. (relation):
 *     I[n] = || (z - z_without_n) W_O ||_2 .
 * If aux_A / aux_ub are not NULL they receive, per (h,i,n), A[n] and the bound
 * A/(1-A) * (||z W_O|| + ||v_n W_O||) used by tests to scale tolerances.
 */
int rk_oracle_indicator_closed(const float* q, const int64_t* qpos, const float* k,
                               const float* v, const double* fac, int r_dim, int G,
                               int nq, int d, int64_t L, int64_t P, double scale,
                               double* I, double* aux_A, double* aux_ub) {
  if (!q || !k || !v || !I || G <= 0 || nq <= 0 || d <= 0 || P < 0 || P > L) return RK_EINVAL;
  if (!fac) r_dim = d;
  int rc = RK_OK;
  for (int h = 0; h < G && rc == RK_OK; ++h) {
    const double* fh = fac ? fac + (int64_t)h * d * r_dim : NULL;
    /* y_n = v_n W_O for every token, once per query head */
    double* y = (double*)malloc(sizeof(double) * (size_t)L * (size_t)r_dim);
    double* ynorm = (double*)malloc(sizeof(double) * (size_t)L);
    if (!y || !ynorm) { free(y); free(ynorm); return RK_ENOMEM; }
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < L; ++n) {
      double vd[1024];
      double* vv = d <= 1024 ? vd : (double*)malloc(sizeof(double) * (size_t)d);
      for (int c = 0; c < d; ++c) vv[c] = (double)v[n * d + c];
      project(vv, fh, d, r_dim, y + n * r_dim);
      double s2 = 0.0;
      for (int r = 0; r < r_dim; ++r) s2 += y[n * r_dim + r] * y[n * r_dim + r];
      ynorm[n] = sqrt(s2);
      if (vv != vd) free(vv);
    }
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < nq; ++i) {
      const int64_t hq = (int64_t)h * nq + i;
      const int64_t nvis = (qpos && qpos[i] >= 0) ? qpos[i] + 1 : L;
      double* e = (double*)malloc(sizeof(double) * (size_t)L);
      double* sl = (double*)malloc(sizeof(double) * (size_t)L);
      double* z = (double*)malloc(sizeof(double) * (size_t)d);
      double* zx = (double*)malloc(sizeof(double) * (size_t)d);
      double* yz = (double*)malloc(sizeof(double) * (size_t)r_dim);
      double* yx = (double*)malloc(sizeof(double) * (size_t)r_dim);
      if (!e || !sl || !z || !zx || !yz || !yx) {
        rc = RK_ENOMEM;
      } else {
        double l;
        softmax_row(q + hq * d, k, d, nvis, scale, e, &l, sl);
        for (int c = 0; c < d; ++c) z[c] = 0.0;
        for (int64_t n = 0; n < nvis; ++n) {
          const double a = e[n] / l;
          for (int c = 0; c < d; ++c) z[c] += a * (double)v[n * d + c];
        }
        project(z, fh, d, r_dim, yz);                 /* MHA output, Eq. (mha) */
        double yznorm = 0.0;
        for (int r = 0; r < r_dim; ++r) yznorm += yz[r] * yz[r];
        yznorm = sqrt(yznorm);
        for (int64_t n = 0; n < P; ++n) {
          double val, a = 0.0, ub = 0.0;
          if (n >= nvis || nvis == 1) {
            val = 0.0;
          } else {
            a = e[n] / l;
            const double rest = l - e[n];             /* sum of the other weights */
            if (2.0 * e[n] <= l) {
              val = e[n] / rest * norm2(yz, y + n * r_dim, r_dim);
            } else {
              /* dominant token: Eq. (ori); softmax over the remaining keys
                 taken afresh from the logits (equal to Eq. (relation)) */
              double mxx = -INFINITY, lx = 0.0;
              for (int64_t m = 0; m < nvis; ++m) if (m != n && sl[m] > mxx) mxx = sl[m];
              for (int64_t m = 0; m < nvis; ++m) if (m != n) lx += exp(sl[m] - mxx);
              for (int c = 0; c < d; ++c) zx[c] = 0.0;
              for (int64_t m = 0; m < nvis; ++m) {
                if (m == n) continue;
                const double am = exp(sl[m] - mxx) / lx;
                for (int c = 0; c < d; ++c) zx[c] += am * (double)v[m * d + c];
              }
              project(zx, fh, d, r_dim, yx);
              val = norm2(yz, yx, r_dim);
            }
            ub = (rest > 0.0 ? e[n] / rest : INFINITY) * (yznorm + ynorm[n]);
          }
          I[hq * P + n] = val;
          if (aux_A) aux_A[hq * P + n] = a;
          if (aux_ub) aux_ub[hq * P + n] = ub;
        }
      }
      free(e); free(sl); free(z); free(zx); free(yz); free(yx);
    }
    free(y); free(ynorm);
  }
  return rc;
}

/*
 * Grouped-query reduction (design reading; the paper treats one head at a
 * time): the G query heads that read one KV head contribute the mean of their
 * indicators, taken before any smoothing.  I [G,nq,P] -> Ig [nq,P].
 */
int rk_oracle_group_mean(const double* I, int G, int nq, int64_t P, double* Ig) {
  if (!I || !Ig || G <= 0 || nq <= 0 || P < 0) return RK_EINVAL;
  for (int64_t x = 0; x < (int64_t)nq * P; ++x) {
    double s = 0.0;
    for (int h = 0; h < G; ++h) s += I[(int64_t)h * nq * P + x];
    Ig[x] = s / (double)G;
  }
  return RK_OK;
}

/*
 * EMA temporal smoothing over the W window queries, by the recursion of
 * Sec. 3.3: EMA over the first query is its indicator; each later query t2
 * enters with weight alpha and the running value keeps (1 - alpha).
 * Ig [W,P] (row i = i-th window query, oldest first) -> ema [P].
 */
int rk_oracle_ema(const double* Ig, int W, int64_t P, double alpha, double* ema) {
  if (!Ig || !ema || W < 1 || P < 0) return RK_EINVAL;
  for (int64_t n = 0; n < P; ++n) {
    double e = Ig[n];
    for (int i = 1; i < W; ++i) e = alpha * Ig[(int64_t)i * P + n] + (1.0 - alpha) * e;
    ema[n] = e;
  }
  return RK_OK;
}

/* order for every top-k here: larger value first, equal values by lower index */
typedef struct { double v; int64_t i; } rk_pair;
static int cmp_desc(const void* a, const void* b) {
  const rk_pair* x = (const rk_pair*)a;
  const rk_pair* y = (const rk_pair*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return x->i < y->i ? -1 : (x->i > y->i ? 1 : 0);
}
static int cmp_i64(const void* a, const void* b) {
  const int64_t x = *(const int64_t*)a, y = *(const int64_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

/* indices of the kk largest entries of s[0..P), ascending; full sort */
static int topk_sorted(const double* s, int64_t P, int64_t kk, int64_t* out) {
  rk_pair* pr = (rk_pair*)malloc(sizeof(rk_pair) * (size_t)(P > 0 ? P : 1));
  if (!pr) return RK_ENOMEM;
  for (int64_t n = 0; n < P; ++n) { pr[n].v = s[n]; pr[n].i = n; }
  qsort(pr, (size_t)P, sizeof(rk_pair), cmp_desc);
  for (int64_t j = 0; j < kk; ++j) out[j] = pr[j].i;
  qsort(out, (size_t)kk, sizeof(int64_t), cmp_i64);
  free(pr);
  return RK_OK;
}

/*
 * Drift statistic of the adaptive window (Sec. 3.3, D_front / D_rear): the mean
 * index of the top-B tokens of each window query, averaged over the first half
 * of the queries (front) and over the remaining ones (rear).  The per-query
 * top-B is taken on the un-smoothed indicator over the P prefix tokens, with
 * Bt = min(B, P) indices per query.  Index sums are also returned as integers.
 */
int rk_oracle_aws_stats(const double* Ig, int W, int64_t P, int64_t B, double* d_front,
                        double* d_rear, int64_t* sum_front, int64_t* sum_rear) {
  if (!Ig || W < 1 || P < 1 || B < 1) return RK_EINVAL;
  const int64_t Bt = B < P ? B : P;
  const int nf = W / 2;
  int64_t sf = 0, sr = 0;
  int64_t* idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)Bt);
  if (!idx) return RK_ENOMEM;
  for (int i = 0; i < W; ++i) {
    int rc = topk_sorted(Ig + (int64_t)i * P, P, Bt, idx);
    if (rc) { free(idx); return rc; }
    int64_t s = 0;
    for (int64_t j = 0; j < Bt; ++j) s += idx[j];
    if (i < nf) sf += s; else sr += s;
  }
  free(idx);
  if (sum_front) *sum_front = sf;
  if (sum_rear) *sum_rear = sr;
  if (d_front) *d_front = nf > 0 ? (double)sf / ((double)Bt * nf) : 0.0;
  if (d_rear) *d_rear = (double)sr / ((double)Bt * (W - nf));
  return RK_OK;
}

/*
 * Window size and shift of the adaptive window (Sec. 3.3):
 *   W_s   = 2 floor(|D_rear - D_front| / beta) + 1      (for base kernel k = 1)
 *   gamma = floor((D_front - D_rear) / beta)            if D_front - D_rear > 0
 *           floor((D_front - D_rear) / beta) + 1        otherwise.
 * Design reading for the fixed kernel size k of App. B: the base window k
 * widens by the same amount, W_s = k + 2 floor(|dD| / beta).  With adaptive = 0
 * the window is k and the shift 0.
 */
int rk_oracle_aws_window(double d_front, double d_rear, double beta, int base_k,
                         int adaptive, int64_t* w_s, int64_t* gamma) {
  if (!w_s || !gamma || base_k < 1 || !(base_k & 1)) return RK_EINVAL;
  if (!adaptive) { *w_s = base_k; *gamma = 0; return RK_OK; }
  if (!(beta > 0.0)) return RK_EINVAL;
  const double x = d_front - d_rear;
  *w_s = (int64_t)base_k + 2 * (int64_t)floor(fabs(x) / beta);
  const int64_t f = (int64_t)floor(x / beta);
  *gamma = x > 0.0 ? f : f + 1;
  return RK_OK;
}

/*
 * Final indicator, Eq. (final_ei): mean over the W_s positions
 * n + gamma - floor(W_s/2) .. n + gamma + floor(W_s/2) of the EMA indicator;
 * positions outside the prefix [0,P) contribute zero and the divisor stays W_s
 * (the window tokens carry no number, they are kept unconditionally).
 */
int rk_oracle_box(const double* ema, int64_t P, int64_t w_s, int64_t gamma, double* out) {
  if (!ema || !out || w_s < 1 || !(w_s & 1)) return RK_EINVAL;
  const int64_t half = w_s / 2;
  for (int64_t n = 0; n < P; ++n) {
    double s = 0.0;
    for (int64_t j = gamma - half; j <= gamma + half; ++j) {
      const int64_t m = n + j;
      if (m >= 0 && m < P) s += ema[m];
    }
    out[n] = s / (double)w_s;
  }
  return RK_OK;
}

/*
 * Selection, Eq. (topk): the B - W prefix tokens with the largest final
 * indicator (equal values: lower index first), in ascending position order,
 * followed by the W window tokens P .. L-1.  idx [B].
 */
int rk_oracle_select(const double* score, int64_t P, int64_t W, int64_t B, int64_t* idx) {
  if (!score || !idx || B <= W || B > P + W) return RK_EINVAL;
  const int64_t Bp = B - W;
  int rc = topk_sorted(score, P, Bp, idx);
  if (rc) return rc;
  for (int64_t j = 0; j < W; ++j) idx[Bp + j] = P + j;
  return RK_OK;
}

/* Gather of the kept rows, Eq. (topk): out[j,:] = src[idx[j],:]; rows of d floats */
int rk_oracle_gather(const float* src, const int64_t* idx, int64_t B, int d, float* out) {
  if (!src || !idx || !out) return RK_EINVAL;
  for (int64_t j = 0; j < B; ++j)
    memcpy(out + j * d, src + idx[j] * (int64_t)d, sizeof(float) * (size_t)d);
  return RK_OK;
}

/* ------------------------------------------------------------------------- */
/* Ablation variants (Sec. 4, ablation table; App. on the ablation study).     */

/*
 * Indicators the paper compares its own with (App., table on the information
 * the indicator considers): the attention weight itself, A[n] ("attention
 * weights"), or the attention weight times the l2 norm of the token's value
 * row, A[n] * ||v_n||_2 ("attention weights and values").  Same argument layout
 * as rk_oracle_indicator_closed; no output projection enters.
 */
int rk_oracle_indicator_attention(const float* q, const int64_t* qpos, const float* k,
                                  const float* v, int G, int nq, int d, int64_t L, int64_t P,
                                  double scale, int value_norm, double* I) {
  if (!q || !k || !v || !I || G <= 0 || nq <= 0 || d <= 0 || P < 0 || P > L) return RK_EINVAL;
  int rc = RK_OK;
#pragma omp parallel for schedule(dynamic)
  for (int64_t hq = 0; hq < (int64_t)G * nq; ++hq) {
    const int64_t i = hq % nq;
    const int64_t nvis = (qpos && qpos[i] >= 0) ? qpos[i] + 1 : L;
    double* e = (double*)malloc(sizeof(double) * (size_t)L);
    if (!e) { rc = RK_ENOMEM; continue; }
    double l;
    softmax_row(q + hq * d, k, d, nvis, scale, e, &l, NULL);
    for (int64_t n = 0; n < P; ++n) {
      double val = n < nvis ? e[n] / l : 0.0;
      if (value_norm) {
        double s2 = 0.0;
        for (int c = 0; c < d; ++c) s2 += (double)v[n * d + c] * (double)v[n * d + c];
        val *= sqrt(s2);
      }
      I[hq * P + n] = val;
    }
    free(e);
  }
  return rc;
}

/* Alternative GQA reduction: the largest indicator among the group's query heads. */
int rk_oracle_group_max(const double* I, int G, int nq, int64_t P, double* Ig) {
  if (!I || !Ig || G <= 0 || nq <= 0 || P < 0) return RK_EINVAL;
  for (int64_t x = 0; x < (int64_t)nq * P; ++x) {
    double m = I[x];
    for (int h = 1; h < G; ++h) if (I[(int64_t)h * nq * P + x] > m) m = I[(int64_t)h * nq * P + x];
    Ig[x] = m;
  }
  return RK_OK;
}

/*
 * Temporal smoothing alternatives (App., table on smoothing methods):
 *   mode 0  EMA, the recursion of Sec. 3.3 (rk_oracle_ema);
 *   mode 1  Mean: the plain average over the W window queries;
 *   mode 2  Inv-EMA: the same recursion run from the newest query to the oldest,
 *           so that the OLDEST query ends with weight alpha and the newest with
 *           (1 - alpha)^(W-1) (the paper does not spell the variant out).
 */
int rk_oracle_temporal(const double* Ig, int W, int64_t P, int mode, double alpha, double* out) {
  if (!Ig || !out || W < 1 || P < 0 || mode < 0 || mode > 2) return RK_EINVAL;
  if (mode == 0) return rk_oracle_ema(Ig, W, P, alpha, out);
  for (int64_t n = 0; n < P; ++n) {
    if (mode == 1) {
      double s = 0.0;
      for (int i = 0; i < W; ++i) s += Ig[(int64_t)i * P + n];
      out[n] = s / (double)W;
    } else {
      double e = Ig[(int64_t)(W - 1) * P + n];
      for (int i = W - 2; i >= 0; --i) e = alpha * Ig[(int64_t)i * P + n] + (1.0 - alpha) * e;
      out[n] = e;
    }
  }
  return RK_OK;
}

/*
 * Max pooling as the spatial smoothing alternative: the largest smoothed
 * indicator among the W_s positions n + gamma - floor(W_s/2) .. n + gamma +
 * floor(W_s/2) that lie inside the prefix (0 if none does).
 */
int rk_oracle_pool_max(const double* ema, int64_t P, int64_t w_s, int64_t gamma, double* out) {
  if (!ema || !out || w_s < 1 || !(w_s & 1)) return RK_EINVAL;
  const int64_t half = w_s / 2;
  for (int64_t n = 0; n < P; ++n) {
    double m = 0.0;
    int any = 0;
    for (int64_t j = gamma - half; j <= gamma + half; ++j) {
      const int64_t x = n + j;
      if (x < 0 || x >= P) continue;
      if (!any || ema[x] > m) m = ema[x];
      any = 1;
    }
    out[n] = m;
  }
  return RK_OK;
}

