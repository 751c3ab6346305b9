/*
 * Reference oracle for Stochastic Attention (SA): a plain, slow, fp64 CPU
 * implementation used ONLY as test infrastructure (tests, the smoke check and
 * the reported CPU baseline of the benchmark).  It shares no code with the
 * HIP library and the HIP library never calls it.
 *
 * Conventions (paper notation in brackets):
 *   perm[p]  = original index of the token that sits at permuted slot p
 *              [the index tensor of "Q[sigma]" in Sec. 3.3; sigma^{-1} of Eq. 3]
 *   inv[i]   = slot of original token i                     [sigma(i) of Eq. 3]
 *   Q  [B,Hq,n,d], K,V [B,Hkv,n,d], row-major doubles; kv head = hq / (Hq/Hkv)
 *   perm [perm_B, perm_H, n] int32, perm_B in {1,B}, perm_H in {1,Hq};
 *        NULL means the identity permutation (plain windowed attention, Eq. 1)
 *   LSE [B,Hq,n] natural-log sum of exp of the scaled scores over the visible set
 *
 * Visible set of query i (Eq. 3, Sec. 3.3 causal paragraph, App. B mask):
 *   { j : window(inv[i], inv[j])  and  (not causal  or  j <= i) }
 * with window(s,t) one of
 *   ORC_WIN_SYM_CIRCULAR  2*min(|s-t|, n-|s-t|) < w      (Sec. 3.1, App. B)
 *   ORC_WIN_SYM_LINEAR    2*|s-t| < w                    (same, without wrap)
 *   ORC_WIN_ONE_SIDED     0 <= s-t <= w-1                (Sec. 3.1 footnote)
 */
#ifndef SA_ORACLE_H
#define SA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_WIN_SYM_CIRCULAR = 0, ORC_WIN_SYM_LINEAR = 1, ORC_WIN_ONE_SIDED = 2 };

typedef struct {
  int32_t B, Hq, Hkv, n, d;
  int32_t w;        /* window size (>= 1, may exceed n)                       */
  int32_t window;   /* ORC_WIN_*                                              */
  int32_t causal;   /* 1: keys must not come after the query in ORIGINAL order */
  int32_t perm_B, perm_H;
  double  scale;    /* softmax scale; <= 0 means 1/sqrt(d) (Eq. 1)             */
} orc_desc;

/* Threads the OpenMP loops will use. */
int orc_num_threads(void);

/* Alg. 1 written out: materialise P_sigma Q, P_sigma K, P_sigma V, run windowed
 * attention over slots, put the rows back.  Y [B,Hq,n,d], LSE [B,Hq,n] (may be
 * NULL).  Returns 0, or a negative value on invalid arguments. */
int orc_sa_fwd(const orc_desc* c, const double* Q, const double* K, const double* V,
               const int32_t* perm, double* Y, double* LSE);

/* Same result for selected rows only, computed straight from the visible-set
 * definition (Eq. 3 / Eq. 4 row by row, no permuted copies).  rows[3*r+0..2] =
 * (b, hq, i).  Y_rows [nrows,d], LSE_rows [nrows] (may be NULL). */
int orc_sa_fwd_rows(const orc_desc* c, const double* Q, const double* K, const double* V,
                    const int32_t* perm, const int32_t* rows, int64_t nrows,
                    double* Y_rows, double* LSE_rows);

/* Number of visible keys of every query: cnt [B,Hq,n] (int64).  Used for the
 * mask statistics of Prop. 1 and for exact "useful flop" counts. */
int orc_visible_count(const orc_desc* c, const int32_t* perm, int64_t* cnt);

/* Eq. 5 with the gate LOGITS given: Y = sig(gsa)*Ysa + sig(gswa)*Yswa.
 * gate_per_dim = 0: logits [B,Hq,n]; 1: logits [B,Hq,n,d]. */
int orc_gate_combine(const orc_desc* c, int gate_per_dim,
                     const double* Ysa, const double* Yswa,
                     const double* gsa, const double* gswa, double* Y);

/* Alg. 2 without the gate projection: both branches then Eq. 5.  `sa` and `swa`
 * describe the two masks (shapes must agree).  Ysa/Yswa/LSEsa/LSEswa may be NULL. */
int orc_gated_sa_swa_fwd(const orc_desc* sa, const orc_desc* swa, int gate_per_dim,
                         const double* Q, const double* K, const double* V,
                         const int32_t* perm, const double* gsa, const double* gswa,
                         double* Y, double* Ysa, double* Yswa,
                         double* LSEsa, double* LSEswa);

/* Gradient of orc_sa_fwd w.r.t. Q, K, V given dY (analytic softmax-attention
 * gradient of Eq. 1 over the visible set).  Outputs are overwritten. */
int orc_sa_bwd(const orc_desc* c, const double* Q, const double* K, const double* V,
               const int32_t* perm, const double* dY,
               double* dQ, double* dK, double* dV);

/* Gradient of orc_gated_sa_swa_fwd w.r.t. Q, K, V and both gate logits. */
int orc_gated_sa_swa_bwd(const orc_desc* sa, const orc_desc* swa, int gate_per_dim,
                         const double* Q, const double* K, const double* V,
                         const int32_t* perm, const double* gsa, const double* gswa,
                         const double* dY,
                         double* dQ, double* dK, double* dV,
                         double* dgsa, double* dgswa);

/* Chain rule through Eq. 5 alone (element-wise): dYsa = sig(gsa)*dY, dYswa = sig(gswa)*dY and, when
 * dgsa/dgswa/Ysa/Yswa are given, the gate-logit gradients.  Works on any set of rows presented as
 * [B,Hq,n,d]. */
int orc_gate_bwd(const orc_desc* c, int gate_per_dim, const double* dY,
                 const double* gsa, const double* gswa, const double* Ysa, const double* Yswa,
                 double* dYsa, double* dYswa, double* dgsa, double* dgswa);

/* Row-sampled gradients for sizes where the full backward is too slow.
 * dQ rows: rows[3*r..] = (b,hq,i) -> dQ_rows [nrows,d].
 * dK/dV rows: rows[3*r..] = (b,hk,j) -> dK_rows, dV_rows [nrows,d]
 * (sum over the Hq/Hkv query heads of the group).  dY is the gradient w.r.t.
 * this branch's own output. */
int orc_sa_bwd_dq_rows(const orc_desc* c, const double* Q, const double* K, const double* V,
                       const int32_t* perm, const double* dY,
                       const int32_t* rows, int64_t nrows, double* dQ_rows);
int orc_sa_bwd_dkv_rows(const orc_desc* c, const double* Q, const double* K, const double* V,
                        const int32_t* perm, const double* dY,
                        const int32_t* rows, int64_t nrows, double* dK_rows, double* dV_rows);

/* Gate projections of the dual-path layer, Eq. 6 followed by Eq. 5 (Alg. 2, "Gated
 * Combination").  Per token t = (b, i) let y_x[t] in R^{dm}, dm = Hq*d, be the
 * concatenation over heads of Y_x[b,h,i,:].  Then
 *   logit_x[t,:] = W_x y_x[t]     (W_x [dm,dm] row-major, row = output feature)
 *   g_x = sigmoid(logit_x),   Y[t,:] = g_sa * y_sa[t] + g_swa * y_swa[t]   (element-wise)
 * Y, Y_sa, Y_swa and the optional logit outputs L_sa, L_swa are [B,Hq,n,d] (feature
 * (h,e) of a token lives at [b,h,i,e]).  Y_swa = W_swa = NULL selects the
 * single-path attention gate of App. B: Y = sigmoid(W_sa y_sa) * y_sa. */
int orc_gate_proj_fwd(const orc_desc* c, const double* Ysa, const double* Yswa,
                      const double* Wsa, const double* Wswa, double* Y, double* Lsa, double* Lswa);

/* Gradient of orc_gate_proj_fwd with respect to the branch outputs and the weights, given dY:
 *   dz_x = dY * y_x * g_x * (1 - g_x),   dy_x = dY * g_x + W_x^T dz_x,   dW_x = sum_t dz_x[t] y_x[t]^T
 * (g_x recomputed from y_x and W_x).  dYsa, dYswa [B,Hq,n,d]; dWsa, dWswa [dm,dm].  The *swa
 * arguments are all NULL for the single path. */
int orc_gate_proj_bwd(const orc_desc* c, const double* Ysa, const double* Yswa,
                      const double* Wsa, const double* Wswa, const double* dY,
                      double* dYsa, double* dYswa, double* dWsa, double* dWswa);

/* Decoding step of the inference setting (Sec. 4.2): one query row per (b, hq) attends to rows
 * 0..len-1 of the K/V caches with plain softmax attention (Eq. 1, every cached row visible).
 * q [B,Hq,d], K,V [B,Hkv,n,d] with n the capacity, 1 <= len <= n, Y [B,Hq,d], LSE [B,Hq] (may be
 * NULL).  w, window, causal and the perm fields of the descriptor are not used. */
int orc_decode_fwd(const orc_desc* c, const double* q, const double* K, const double* V,
                   int32_t len, double* Y, double* LSE);

#ifdef __cplusplus
}
#endif
#endif
