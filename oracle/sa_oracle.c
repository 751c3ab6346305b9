/*
 * Reference oracle for Stochastic Attention -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 loops written from the paper's definitions.  Nothing here is
 * blocked, fused or tuned; nothing here is shared with (or called by) the HIP
 * library.  See sa_oracle.h for conventions.  Each function names the passage
 * it follows.
 */
#include "sa_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ helpers */

static int desc_ok(const orc_desc* c) {
  if (!c) return 0;
  if (c->B < 1 || c->Hq < 1 || c->Hkv < 1 || c->n < 1 || c->d < 1 || c->w < 1) return 0;
  if (c->Hq % c->Hkv != 0) return 0;
  if (c->window < 0 || c->window > 2) return 0;
  if (!(c->perm_B == 1 || c->perm_B == c->B)) return 0;
  if (!(c->perm_H == 1 || c->perm_H == c->Hq)) return 0;
  return 1;
}

static double softmax_scale(const orc_desc* c) {
  return c->scale > 0.0 ? c->scale : 1.0 / sqrt((double)c->d); /* Eq. 1: 1/sqrt(d_h) */
}

/* Window predicate on two SLOTS, literally as printed:
 *   circular symmetric  |s-t|_n < w/2 with |x|_n = min(|x|, n-|x|)  (Sec. 3.1; App. B mask)
 *   linear symmetric    |s-t| < w/2
 *   one-sided           0 <= s-t <= w-1                             (Sec. 3.1 footnote)
 * "< w/2" is evaluated in integers as 2*dist < w. */
static int in_window(const orc_desc* c, int64_t s, int64_t t) {
  int64_t n = c->n, w = c->w;
  int64_t diff = s - t;
  int64_t a = diff < 0 ? -diff : diff;
  if (c->window == ORC_WIN_SYM_CIRCULAR) {
    int64_t circ = a < n - a ? a : n - a;
    return 2 * circ < w;
  }
  if (c->window == ORC_WIN_SYM_LINEAR) return 2 * a < w;
  return diff >= 0 && diff <= w - 1;
}

/* Candidate slots around slot s: a superset of every window kind's support
 * (|s-t| <= w, wrapped), each slot listed once.  The caller still applies
 * in_window() to every candidate; this only avoids scanning all n slots. */
static int64_t candidate_slots(const orc_desc* c, int64_t s, int32_t* out) {
  int64_t n = c->n, r = c->w, m = 0;
  if (2 * r + 1 >= n) {
    for (int64_t t = 0; t < n; ++t) out[m++] = (int32_t)t;
    return m;
  }
  for (int64_t dlt = -r; dlt <= r; ++dlt) {
    int64_t t = s + dlt;
    if (c->window == ORC_WIN_SYM_CIRCULAR) {
      t %= n;
      if (t < 0) t += n;
    } else if (t < 0 || t >= n) {
      continue;
    }
    out[m++] = (int32_t)t;
  }
  return m;
}

static const int32_t* perm_slice(const orc_desc* c, const int32_t* perm, int b, int hq) {
  if (!perm) return NULL;
  int64_t pb = c->perm_B == 1 ? 0 : b;
  int64_t ph = c->perm_H == 1 ? 0 : hq;
  return perm + (pb * c->perm_H + ph) * (int64_t)c->n;
}

/* inverse of every distinct permutation: inv[perm[p]] = p.  Returns NULL with
 * *bad = 1 when some slice is not a bijection of 0..n-1. */
static int32_t* build_inverses(const orc_desc* c, const int32_t* perm, int* bad) {
  *bad = 0;
  if (!perm) return NULL;
  int64_t n = c->n, np = (int64_t)c->perm_B * c->perm_H;
  int32_t* inv = (int32_t*)malloc(sizeof(int32_t) * (size_t)(np * n));
  if (!inv) { *bad = 1; return NULL; }
  for (int64_t k = 0; k < np * n; ++k) inv[k] = -1;
  for (int64_t q = 0; q < np && !*bad; ++q) {
    for (int64_t p = 0; p < n; ++p) {
      int32_t i = perm[q * n + p];
      if (i < 0 || i >= n || inv[q * n + i] != -1) { *bad = 1; break; }
      inv[q * n + i] = (int32_t)p;
    }
  }
  if (*bad) { free(inv); return NULL; }
  return inv;
}

static double dot(const double* a, const double* b, int d) {
  double s = 0.0;
  for (int k = 0; k < d; ++k) s += a[k] * b[k];
  return s;
}

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); } /* exact 0/1 at -inf/+inf */

/* ------------------------------------------------- Alg. 1, written out whole */

int orc_sa_fwd(const orc_desc* c, const double* Q, const double* K, const double* V,
               const int32_t* perm, double* Y, double* LSE) {
  if (!desc_ok(c) || !Q || !K || !V || !Y) return -1;
  int bad = 0;
  int32_t* inv_check = build_inverses(c, perm, &bad); /* only validates here */
  if (bad) return -2;
  free(inv_check);

  const int64_t n = c->n;
  const int d = c->d, g = c->Hq / c->Hkv;
  const double scale = softmax_scale(c);
  double* Qt = (double*)malloc(sizeof(double) * (size_t)(n * d));
  double* Kt = (double*)malloc(sizeof(double) * (size_t)(n * d));
  double* Vt = (double*)malloc(sizeof(double) * (size_t)(n * d));
  double* Yt = (double*)malloc(sizeof(double) * (size_t)(n * d));
  double* Lt = (double*)malloc(sizeof(double) * (size_t)n);
  int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  if (!Qt || !Kt || !Vt || !Yt || !Lt || !pos) return -3;

  for (int b = 0; b < c->B; ++b) {
    for (int hq = 0; hq < c->Hq; ++hq) {
      const int hk = hq / g;
      const double* Qh = Q + ((int64_t)b * c->Hq + hq) * n * d;
      const double* Kh = K + ((int64_t)b * c->Hkv + hk) * n * d;
      const double* Vh = V + ((int64_t)b * c->Hkv + hk) * n * d;
      double* Yh = Y + ((int64_t)b * c->Hq + hq) * n * d;
      const int32_t* pm = perm_slice(c, perm, b, hq);

      /* line "permute": X~ = P_sigma X, i.e. row p of X~ is row perm[p] of X */
      for (int64_t p = 0; p < n; ++p) {
        int64_t src = pm ? pm[p] : p;
        pos[p] = (int32_t)src; /* original position carried along for the causal test */
        memcpy(Qt + p * d, Qh + src * d, sizeof(double) * (size_t)d);
        memcpy(Kt + p * d, Kh + src * d, sizeof(double) * (size_t)d);
        memcpy(Vt + p * d, Vh + src * d, sizeof(double) * (size_t)d);
      }

      /* line "windowed attention in permuted space": Eq. 1 over slots, with the
       * causal constraint of Sec. 3.3 evaluated on original positions */
#pragma omp parallel
      {
        int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
        double* z = (double*)malloc(sizeof(double) * (size_t)n);
        int32_t* keep = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
#pragma omp for schedule(static)
        for (int64_t p = 0; p < n; ++p) {
          int64_t nc = candidate_slots(c, p, cand), m = 0;
          for (int64_t a = 0; a < nc; ++a) {
            int64_t t = cand[a];
            if (!in_window(c, p, t)) continue;
            if (c->causal && pos[t] > pos[p]) continue;
            keep[m] = (int32_t)t;
            z[m] = scale * dot(Qt + p * d, Kt + t * d, d);
            ++m;
          }
          double zmax = -INFINITY, sum = 0.0;
          for (int64_t a = 0; a < m; ++a) if (z[a] > zmax) zmax = z[a];
          for (int64_t a = 0; a < m; ++a) sum += exp(z[a] - zmax);
          double* y = Yt + p * d;
          for (int k = 0; k < d; ++k) y[k] = 0.0;
          for (int64_t a = 0; a < m; ++a) {
            double alpha = exp(z[a] - zmax) / sum;
            const double* v = Vt + (int64_t)keep[a] * d;
            for (int k = 0; k < d; ++k) y[k] += alpha * v[k];
          }
          Lt[p] = zmax + log(sum);
        }
        free(cand); free(z); free(keep);
      }

      /* line "undo permute": Y = P_{sigma^-1} Y~, i.e. row perm[p] of Y is row p of Y~ */
      for (int64_t p = 0; p < n; ++p) {
        memcpy(Yh + (int64_t)pos[p] * d, Yt + p * d, sizeof(double) * (size_t)d);
        if (LSE) LSE[((int64_t)b * c->Hq + hq) * n + pos[p]] = Lt[p];
      }
    }
  }
  free(Qt); free(Kt); free(Vt); free(Yt); free(Lt); free(pos);
  return 0;
}

/* ------------------------------- row-wise form straight from the visible set */

/* Visible keys of query i (original indices) with their attention weights.
 * js/ps must hold n entries.  Returns the count; *lse = log-sum-exp. */
static int64_t softmax_row(const orc_desc* c, const double* Q, const double* K,
                           const int32_t* pm, const int32_t* iv, int b, int hq, int64_t i,
                           int32_t* cand, int32_t* js, double* ps, double* lse) {
  const int64_t n = c->n;
  const int d = c->d, hk = hq / (c->Hq / c->Hkv);
  const double scale = softmax_scale(c);
  const double* q = Q + (((int64_t)b * c->Hq + hq) * n + i) * d;
  const double* Kh = K + ((int64_t)b * c->Hkv + hk) * n * d;
  int64_t s = iv ? iv[i] : i; /* sigma(i) */
  int64_t nc = candidate_slots(c, s, cand), m = 0;
  for (int64_t a = 0; a < nc; ++a) {
    int64_t t = cand[a];
    int64_t j = pm ? pm[t] : t; /* sigma^{-1}(t) */
    if (!in_window(c, s, t)) continue;     /* Eq. 3 */
    if (c->causal && j > i) continue;      /* Sec. 3.3: only j <= i */
    js[m] = (int32_t)j;
    ps[m] = scale * dot(q, Kh + j * d, d);
    ++m;
  }
  double zmax = -INFINITY, sum = 0.0;
  for (int64_t a = 0; a < m; ++a) if (ps[a] > zmax) zmax = ps[a];
  for (int64_t a = 0; a < m; ++a) sum += exp(ps[a] - zmax);
  for (int64_t a = 0; a < m; ++a) ps[a] = exp(ps[a] - zmax) / sum;
  *lse = zmax + log(sum);
  return m;
}

int orc_sa_fwd_rows(const orc_desc* c, const double* Q, const double* K, const double* V,
                    const int32_t* perm, const int32_t* rows, int64_t nrows,
                    double* Y_rows, double* LSE_rows) {
  if (!desc_ok(c) || !Q || !K || !V || !rows || !Y_rows || nrows < 0) return -1;
  int bad = 0;
  int32_t* inv = build_inverses(c, perm, &bad);
  if (bad) return -2;
  const int64_t n = c->n;
  const int d = c->d, g = c->Hq / c->Hkv;
  for (int64_t r = 0; r < nrows; ++r) {
    if (rows[3 * r] < 0 || rows[3 * r] >= c->B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= c->Hq ||
        rows[3 * r + 2] < 0 || rows[3 * r + 2] >= n) { free(inv); return -1; }
  }
#pragma omp parallel
  {
    int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    int32_t* js = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    double* ps = (double*)malloc(sizeof(double) * (size_t)n);
#pragma omp for schedule(dynamic, 16)
    for (int64_t r = 0; r < nrows; ++r) {
      int b = rows[3 * r], hq = rows[3 * r + 1];
      int64_t i = rows[3 * r + 2];
      const int32_t* pm = perm_slice(c, perm, b, hq);
      const int32_t* iv = perm_slice(c, inv, b, hq);
      double lse;
      int64_t m = softmax_row(c, Q, K, pm, iv, b, hq, i, cand, js, ps, &lse);
      const double* Vh = V + ((int64_t)b * c->Hkv + hq / g) * n * d;
      double* y = Y_rows + r * d;
      for (int k = 0; k < d; ++k) y[k] = 0.0;
      for (int64_t a = 0; a < m; ++a) {
        const double* v = Vh + (int64_t)js[a] * d;
        for (int k = 0; k < d; ++k) y[k] += ps[a] * v[k];
      }
      if (LSE_rows) LSE_rows[r] = lse;
    }
    free(cand); free(js); free(ps);
  }
  free(inv);
  return 0;
}

int orc_visible_count(const orc_desc* c, const int32_t* perm, int64_t* cnt) {
  if (!desc_ok(c) || !cnt) return -1;
  int bad = 0;
  int32_t* inv = build_inverses(c, perm, &bad);
  if (bad) return -2;
  const int64_t n = c->n;
#pragma omp parallel
  {
    int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
#pragma omp for collapse(2) schedule(static)
    for (int b = 0; b < c->B; ++b) {
      for (int hq = 0; hq < c->Hq; ++hq) {
        const int32_t* pm = perm_slice(c, perm, b, hq);
        const int32_t* iv = perm_slice(c, inv, b, hq);
        for (int64_t i = 0; i < n; ++i) {
          int64_t s = iv ? iv[i] : i, m = 0;
          int64_t nc = candidate_slots(c, s, cand);
          for (int64_t a = 0; a < nc; ++a) {
            int64_t t = cand[a], j = pm ? pm[t] : t;
            if (in_window(c, s, t) && (!c->causal || j <= i)) ++m;
          }
          cnt[((int64_t)b * c->Hq + hq) * n + i] = m;
        }
      }
    }
    free(cand);
  }
  free(inv);
  return 0;
}

/* ------------------------------------------------------------ Eq. 5 (gates) */

int orc_gate_combine(const orc_desc* c, int gate_per_dim,
                     const double* Ysa, const double* Yswa,
                     const double* gsa, const double* gswa, double* Y) {
  if (!desc_ok(c) || !Ysa || !Yswa || !gsa || !gswa || !Y) return -1;
  const int64_t rows = (int64_t)c->B * c->Hq * c->n;
  const int d = c->d;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    for (int k = 0; k < d; ++k) {
      int64_t e = r * d + k;
      double a = sigmoid(gate_per_dim ? gsa[e] : gsa[r]);
      double l = sigmoid(gate_per_dim ? gswa[e] : gswa[r]);
      Y[e] = a * Ysa[e] + l * Yswa[e];
    }
  }
  return 0;
}

static int same_shape(const orc_desc* a, const orc_desc* b) {
  return a->B == b->B && a->Hq == b->Hq && a->Hkv == b->Hkv && a->n == b->n && a->d == b->d;
}

int orc_gated_sa_swa_fwd(const orc_desc* sa, const orc_desc* swa, int gate_per_dim,
                         const double* Q, const double* K, const double* V,
                         const int32_t* perm, const double* gsa, const double* gswa,
                         double* Y, double* Ysa, double* Yswa,
                         double* LSEsa, double* LSEswa) {
  if (!desc_ok(sa) || !desc_ok(swa) || !same_shape(sa, swa) || !Y) return -1;
  const size_t ne = (size_t)sa->B * sa->Hq * sa->n * sa->d;
  double* ya = Ysa ? Ysa : (double*)malloc(sizeof(double) * ne);
  double* yl = Yswa ? Yswa : (double*)malloc(sizeof(double) * ne);
  if (!ya || !yl) return -3;
  int rc = orc_sa_fwd(sa, Q, K, V, perm, ya, LSEsa);          /* Alg. 2: stochastic branch */
  if (!rc) rc = orc_sa_fwd(swa, Q, K, V, NULL, yl, LSEswa);   /* Alg. 2: sliding-window branch */
  if (!rc) rc = orc_gate_combine(sa, gate_per_dim, ya, yl, gsa, gswa, Y);
  if (!Ysa) free(ya);
  if (!Yswa) free(yl);
  return rc;
}

/* ----------------------------------------------------------------- backward */

/* Gradient of Y_i = sum_j p_ij V_j, p = softmax_j(scale <Q_i,K_j>) over the
 * visible set (Eq. 1): with D_i = <dY_i, Y_i>,
 *   dV_j += p_ij dY_i,   dS_ij = p_ij (<dY_i,V_j> - D_i),
 *   dQ_i += scale dS_ij K_j,   dK_j += scale dS_ij Q_i. */
int orc_sa_bwd(const orc_desc* c, const double* Q, const double* K, const double* V,
               const int32_t* perm, const double* dY,
               double* dQ, double* dK, double* dV) {
  if (!desc_ok(c) || !Q || !K || !V || !dY || !dQ || !dK || !dV) return -1;
  int bad = 0;
  int32_t* inv = build_inverses(c, perm, &bad);
  if (bad) return -2;
  const int64_t n = c->n;
  const int d = c->d, g = c->Hq / c->Hkv;
  const double scale = softmax_scale(c);
  memset(dQ, 0, sizeof(double) * (size_t)c->B * c->Hq * n * d);
  memset(dK, 0, sizeof(double) * (size_t)c->B * c->Hkv * n * d);
  memset(dV, 0, sizeof(double) * (size_t)c->B * c->Hkv * n * d);
  /* one (batch, kv head) per iteration: the only writer of its dK/dV rows */
#pragma omp parallel
  {
    int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    int32_t* js = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    double* ps = (double*)malloc(sizeof(double) * (size_t)n);
    double* y = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < c->B; ++b) {
      for (int hk = 0; hk < c->Hkv; ++hk) {
        const double* Kh = K + ((int64_t)b * c->Hkv + hk) * n * d;
        const double* Vh = V + ((int64_t)b * c->Hkv + hk) * n * d;
        double* dKh = dK + ((int64_t)b * c->Hkv + hk) * n * d;
        double* dVh = dV + ((int64_t)b * c->Hkv + hk) * n * d;
        for (int hq = hk * g; hq < (hk + 1) * g; ++hq) {
          const int32_t* pm = perm_slice(c, perm, b, hq);
          const int32_t* iv = perm_slice(c, inv, b, hq);
          for (int64_t i = 0; i < n; ++i) {
            double lse;
            int64_t m = softmax_row(c, Q, K, pm, iv, b, hq, i, cand, js, ps, &lse);
            const int64_t qoff = (((int64_t)b * c->Hq + hq) * n + i) * d;
            const double* q = Q + qoff;
            const double* dy = dY + qoff;
            double* dq = dQ + qoff;
            for (int k = 0; k < d; ++k) y[k] = 0.0;
            for (int64_t a = 0; a < m; ++a)
              for (int k = 0; k < d; ++k) y[k] += ps[a] * Vh[(int64_t)js[a] * d + k];
            const double D = dot(dy, y, d);
            for (int64_t a = 0; a < m; ++a) {
              const int64_t j = js[a];
              const double dP = dot(dy, Vh + j * d, d);
              const double dS = ps[a] * (dP - D);
              for (int k = 0; k < d; ++k) {
                dVh[j * d + k] += ps[a] * dy[k];
                dq[k] += scale * dS * Kh[j * d + k];
                dKh[j * d + k] += scale * dS * q[k];
              }
            }
          }
        }
      }
    }
    free(cand); free(js); free(ps); free(y);
  }
  free(inv);
  return 0;
}

/* Chain rule through Eq. 5, element-wise: with a = sig(gamma_sa), l = sig(gamma_swa),
 *   dY_sa = a * dY,  dgamma_sa = a(1-a) * dY*Y_sa  (summed over d when the gate is per token),
 * likewise for the sliding-window branch.  Rows are independent, so the tensors may also be any
 * subset of rows presented as [B,Hq,n,d] with matching logits.  Ysa, Yswa, dgsa, dgswa may all be
 * NULL when only dY_sa / dY_swa are wanted. */
int orc_gate_bwd(const orc_desc* c, int gate_per_dim, const double* dY,
                 const double* gsa, const double* gswa, const double* Ysa, const double* Yswa,
                 double* dYsa, double* dYswa, double* dgsa, double* dgswa) {
  if (!desc_ok(c) || !dY || !gsa || !gswa || !dYsa || !dYswa) return -1;
  const int want_dg = dgsa || dgswa;
  if (want_dg && (!dgsa || !dgswa || !Ysa || !Yswa)) return -1;
  const int64_t rows = (int64_t)c->B * c->Hq * c->n;
  const int d = c->d;
  for (int64_t r = 0; r < rows; ++r) {
    double acc_a = 0.0, acc_l = 0.0;
    for (int k = 0; k < d; ++k) {
      int64_t e = r * d + k;
      double a = sigmoid(gate_per_dim ? gsa[e] : gsa[r]);
      double l = sigmoid(gate_per_dim ? gswa[e] : gswa[r]);
      dYsa[e] = a * dY[e];
      dYswa[e] = l * dY[e];
      if (!want_dg) continue;
      if (gate_per_dim) {
        dgsa[e] = a * (1.0 - a) * dY[e] * Ysa[e];
        dgswa[e] = l * (1.0 - l) * dY[e] * Yswa[e];
      } else {
        acc_a += dY[e] * Ysa[e];
        acc_l += dY[e] * Yswa[e];
      }
    }
    if (want_dg && !gate_per_dim) {
      double a = sigmoid(gsa[r]), l = sigmoid(gswa[r]);
      dgsa[r] = a * (1.0 - a) * acc_a;
      dgswa[r] = l * (1.0 - l) * acc_l;
    }
  }
  return 0;
}

/* Gradient of Alg. 2 (with the gate logits as inputs): both branches forward, Eq. 5's chain rule,
 * each branch's attention gradient, and the sum of the two for dQ, dK, dV. */
int orc_gated_sa_swa_bwd(const orc_desc* sa, const orc_desc* swa, int gate_per_dim,
                         const double* Q, const double* K, const double* V,
                         const int32_t* perm, const double* gsa, const double* gswa,
                         const double* dY,
                         double* dQ, double* dK, double* dV,
                         double* dgsa, double* dgswa) {
  if (!desc_ok(sa) || !desc_ok(swa) || !same_shape(sa, swa)) return -1;
  if (!gsa || !gswa || !dY || !dQ || !dK || !dV || !dgsa || !dgswa) return -1;
  const size_t nq = (size_t)sa->B * sa->Hq * sa->n * sa->d, nk = (size_t)sa->B * sa->Hkv * sa->n * sa->d;
  double* ya = (double*)malloc(sizeof(double) * nq);
  double* yl = (double*)malloc(sizeof(double) * nq);
  double* da = (double*)malloc(sizeof(double) * nq);
  double* dl = (double*)malloc(sizeof(double) * nq);
  double* dQ2 = (double*)malloc(sizeof(double) * nq);
  double* dK2 = (double*)malloc(sizeof(double) * nk);
  double* dV2 = (double*)malloc(sizeof(double) * nk);
  if (!ya || !yl || !da || !dl || !dQ2 || !dK2 || !dV2) return -3;
  int rc = orc_sa_fwd(sa, Q, K, V, perm, ya, NULL);
  if (!rc) rc = orc_sa_fwd(swa, Q, K, V, NULL, yl, NULL);
  if (!rc) rc = orc_gate_bwd(sa, gate_per_dim, dY, gsa, gswa, ya, yl, da, dl, dgsa, dgswa);
  if (!rc) rc = orc_sa_bwd(sa, Q, K, V, perm, da, dQ, dK, dV);
  if (!rc) rc = orc_sa_bwd(swa, Q, K, V, NULL, dl, dQ2, dK2, dV2);
  if (!rc) {
    for (size_t e = 0; e < nq; ++e) dQ[e] += dQ2[e];
    for (size_t e = 0; e < nk; ++e) { dK[e] += dK2[e]; dV[e] += dV2[e]; }
  }
  free(ya); free(yl); free(da); free(dl); free(dQ2); free(dK2); free(dV2);
  return rc;
}

int orc_sa_bwd_dq_rows(const orc_desc* c, const double* Q, const double* K, const double* V,
                       const int32_t* perm, const double* dY,
                       const int32_t* rows, int64_t nrows, double* dQ_rows) {
  if (!desc_ok(c) || !Q || !K || !V || !dY || !rows || !dQ_rows || nrows < 0) return -1;
  int bad = 0;
  int32_t* inv = build_inverses(c, perm, &bad);
  if (bad) return -2;
  const int64_t n = c->n;
  const int d = c->d, g = c->Hq / c->Hkv;
  const double scale = softmax_scale(c);
#pragma omp parallel
  {
    int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    int32_t* js = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    double* ps = (double*)malloc(sizeof(double) * (size_t)n);
    double* y = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 16)
    for (int64_t r = 0; r < nrows; ++r) {
      int b = rows[3 * r], hq = rows[3 * r + 1];
      int64_t i = rows[3 * r + 2];
      const int32_t* pm = perm_slice(c, perm, b, hq);
      const int32_t* iv = perm_slice(c, inv, b, hq);
      const double* Kh = K + ((int64_t)b * c->Hkv + hq / g) * n * d;
      const double* Vh = V + ((int64_t)b * c->Hkv + hq / g) * n * d;
      const double* dy = dY + (((int64_t)b * c->Hq + hq) * n + i) * d;
      double lse;
      int64_t m = softmax_row(c, Q, K, pm, iv, b, hq, i, cand, js, ps, &lse);
      for (int k = 0; k < d; ++k) y[k] = 0.0;
      for (int64_t a = 0; a < m; ++a)
        for (int k = 0; k < d; ++k) y[k] += ps[a] * Vh[(int64_t)js[a] * d + k];
      const double D = dot(dy, y, d);
      double* dq = dQ_rows + r * d;
      for (int k = 0; k < d; ++k) dq[k] = 0.0;
      for (int64_t a = 0; a < m; ++a) {
        const double dS = ps[a] * (dot(dy, Vh + (int64_t)js[a] * d, d) - D);
        for (int k = 0; k < d; ++k) dq[k] += scale * dS * Kh[(int64_t)js[a] * d + k];
      }
    }
    free(cand); free(js); free(ps); free(y);
  }
  free(inv);
  return 0;
}

int orc_sa_bwd_dkv_rows(const orc_desc* c, const double* Q, const double* K, const double* V,
                        const int32_t* perm, const double* dY,
                        const int32_t* rows, int64_t nrows, double* dK_rows, double* dV_rows) {
  if (!desc_ok(c) || !Q || !K || !V || !dY || !rows || !dK_rows || !dV_rows || nrows < 0) return -1;
  int bad = 0;
  int32_t* inv = build_inverses(c, perm, &bad);
  if (bad) return -2;
  const int64_t n = c->n;
  const int d = c->d, g = c->Hq / c->Hkv;
  const double scale = softmax_scale(c);
#pragma omp parallel
  {
    int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    int32_t* qcand = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    int32_t* js = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    double* ps = (double*)malloc(sizeof(double) * (size_t)n);
    double* y = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
    for (int64_t r = 0; r < nrows; ++r) {
      int b = rows[3 * r], hk = rows[3 * r + 1];
      int64_t j = rows[3 * r + 2];
      const double* Vh = V + ((int64_t)b * c->Hkv + hk) * n * d;
      double* dk = dK_rows + r * d;
      double* dv = dV_rows + r * d;
      for (int k = 0; k < d; ++k) { dk[k] = 0.0; dv[k] = 0.0; }
      for (int hq = hk * g; hq < (hk + 1) * g; ++hq) {
        const int32_t* pm = perm_slice(c, perm, b, hq);
        const int32_t* iv = perm_slice(c, inv, b, hq);
        /* every query that can see key j sits at a slot near j's slot */
        int64_t t = iv ? iv[j] : j;
        int64_t nq = candidate_slots(c, t, qcand);
        for (int64_t u = 0; u < nq; ++u) {
          int64_t s = qcand[u], i = pm ? pm[s] : s;
          if (!in_window(c, s, t)) continue;
          if (c->causal && j > i) continue;
          double lse;
          int64_t m = softmax_row(c, Q, K, pm, iv, b, hq, i, cand, js, ps, &lse);
          const int64_t qoff = (((int64_t)b * c->Hq + hq) * n + i) * d;
          const double* dy = dY + qoff;
          double pij = 0.0;
          for (int k = 0; k < d; ++k) y[k] = 0.0;
          for (int64_t a = 0; a < m; ++a) {
            if (js[a] == j) pij = ps[a];
            for (int k = 0; k < d; ++k) y[k] += ps[a] * Vh[(int64_t)js[a] * d + k];
          }
          const double D = dot(dy, y, d);
          const double dS = pij * (dot(dy, Vh + j * d, d) - D);
          for (int k = 0; k < d; ++k) {
            dv[k] += pij * dy[k];
            dk[k] += scale * dS * Q[qoff + k];
          }
        }
      }
    }
    free(cand); free(qcand); free(js); free(ps); free(y);
  }
  free(inv);
  return 0;
}

/* ---------------------------------------------------------------- gate projections (Eq. 6, Eq. 5) */
int orc_gate_proj_fwd(const orc_desc* c, const double* Ysa, const double* Yswa,
                      const double* Wsa, const double* Wswa, double* Y, double* Lsa, double* Lswa) {
  if (!desc_ok(c) || !Ysa || !Wsa || !Y) return -1;
  if ((Yswa == NULL) != (Wswa == NULL)) return -1;
  const int64_t n = c->n, d = c->d, H = c->Hq, dm = H * d;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t b = 0; b < c->B; ++b) {
    for (int64_t i = 0; i < n; ++i) {
      for (int64_t o = 0; o < dm; ++o) {            /* output feature o = (ho, eo) */
        const int64_t ho = o / d, eo = o % d;
        const int64_t at = ((b * H + ho) * n + i) * d + eo;
        double za = 0.0, zb = 0.0;
        for (int64_t k = 0; k < dm; ++k) {          /* input feature k = (hk, ek) */
          const int64_t src = ((b * H + k / d) * n + i) * d + k % d;
          za += Wsa[o * dm + k] * Ysa[src];
          if (Yswa) zb += Wswa[o * dm + k] * Yswa[src];
        }
        double y = sigmoid(za) * Ysa[at];
        if (Yswa) y += sigmoid(zb) * Yswa[at];
        Y[at] = y;
        if (Lsa) Lsa[at] = za;
        if (Lswa && Yswa) Lswa[at] = zb;
      }
    }
  }
  return 0;
}

static void gate_proj_bwd_branch(const orc_desc* c, const double* Yx, const double* W, const double* dY,
                                 double* dYx, double* dW) {
  const int64_t n = c->n, d = c->d, H = c->Hq, dm = H * d;
  for (int64_t e = 0; e < dm * dm; ++e) dW[e] = 0.0;
  double* y = (double*)malloc(sizeof(double) * (size_t)dm);   /* one token, features concatenated */
  double* dz = (double*)malloc(sizeof(double) * (size_t)dm);
  double* g = (double*)malloc(sizeof(double) * (size_t)dm);
  for (int64_t b = 0; b < c->B; ++b) {
    for (int64_t i = 0; i < n; ++i) {
      for (int64_t k = 0; k < dm; ++k) y[k] = Yx[((b * H + k / d) * n + i) * d + k % d];
      for (int64_t o = 0; o < dm; ++o) {
        double z = 0.0;
        for (int64_t k = 0; k < dm; ++k) z += W[o * dm + k] * y[k];
        g[o] = sigmoid(z);
        const double dy_o = dY[((b * H + o / d) * n + i) * d + o % d];
        dz[o] = dy_o * y[o] * g[o] * (1.0 - g[o]);
      }
      for (int64_t k = 0; k < dm; ++k) {
        double acc = dY[((b * H + k / d) * n + i) * d + k % d] * g[k];
        for (int64_t o = 0; o < dm; ++o) acc += W[o * dm + k] * dz[o];
        dYx[((b * H + k / d) * n + i) * d + k % d] = acc;
      }
      for (int64_t o = 0; o < dm; ++o)
        for (int64_t k = 0; k < dm; ++k) dW[o * dm + k] += dz[o] * y[k];
    }
  }
  free(y); free(dz); free(g);
}

int orc_gate_proj_bwd(const orc_desc* c, const double* Ysa, const double* Yswa,
                      const double* Wsa, const double* Wswa, const double* dY,
                      double* dYsa, double* dYswa, double* dWsa, double* dWswa) {
  if (!desc_ok(c) || !Ysa || !Wsa || !dY || !dYsa || !dWsa) return -1;
  const int dual = Yswa != NULL;
  if (dual != (Wswa != NULL) || dual != (dYswa != NULL) || dual != (dWswa != NULL)) return -1;
  gate_proj_bwd_branch(c, Ysa, Wsa, dY, dYsa, dWsa);
  if (dual) gate_proj_bwd_branch(c, Yswa, Wswa, dY, dYswa, dWswa);
  return 0;
}

/* ------------------------------------------------------------------ decode */

/* Sec. 4.2 (inference setting): the sparse modes are used while the prompt is
 * processed; each generated token then attends to the WHOLE cache.  One query
 * row per (b, hq), plain softmax attention (Eq. 1 with the window covering
 * every cached row) over rows 0..len-1 of the caches:
 *   z_j = scale <q, K_j>,  LSE = log sum_j e^{z_j},  Y = sum_j e^{z_j - LSE} V_j.
 * q [B,Hq,d], K,V [B,Hkv,n,d] (n = capacity), Y [B,Hq,d], LSE [B,Hq] or NULL. */
int orc_decode_fwd(const orc_desc* c, const double* q, const double* K, const double* V,
                   int32_t len, double* Y, double* LSE) {
  if (!desc_ok(c) || !q || !K || !V || !Y) return -1;
  if (len < 1 || len > c->n) return -2;
  const int g = c->Hq / c->Hkv;
  const double scale = softmax_scale(c);
  for (int b = 0; b < c->B; ++b) {
    for (int hq = 0; hq < c->Hq; ++hq) {
      const int hk = hq / g;
      const double* qr = q + ((size_t)b * c->Hq + hq) * c->d;
      const double* Kh = K + ((size_t)b * c->Hkv + hk) * (size_t)c->n * c->d;
      const double* Vh = V + ((size_t)b * c->Hkv + hk) * (size_t)c->n * c->d;
      double* z = (double*)malloc((size_t)len * sizeof(double));
      if (!z) return -3;
      double zmax = -INFINITY;
      for (int j = 0; j < len; ++j) {
        z[j] = scale * dot(qr, Kh + (size_t)j * c->d, c->d);
        if (z[j] > zmax) zmax = z[j];
      }
      double sum = 0.0;
      for (int j = 0; j < len; ++j) sum += exp(z[j] - zmax);
      const double lse = zmax + log(sum);
      double* y = Y + ((size_t)b * c->Hq + hq) * c->d;
      for (int e = 0; e < c->d; ++e) y[e] = 0.0;
      for (int j = 0; j < len; ++j) {
        const double pj = exp(z[j] - lse);
        for (int e = 0; e < c->d; ++e) y[e] += pj * Vh[(size_t)j * c->d + e];
      }
      if (LSE) LSE[(size_t)b * c->Hq + hq] = lse;
      free(z);
    }
  }
  return 0;
}
