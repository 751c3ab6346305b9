/*
 * libsa -- Stochastic Attention (SA) hot path for AMD MI355X (gfx950), C ABI.
 *
 * What the library computes (paper: "Stochastic Attention", Sec. 3.3, Sec. 3.4, App. B):
 *   SA:   permute tokens with a sampled permutation, run windowed softmax attention in the permuted
 *         order, put the outputs back (Alg. 1).  Equivalently (Eq. 3, Eq. 4) every query i attends to
 *         the keys j whose SLOTS are within the window of i's slot, and -- for causal language
 *         models -- whose ORIGINAL position is not after i (Sec. 3.3, App. B "stochastic attention
 *         mask").
 *   SWA:  the same with the identity permutation (Eq. 1).
 *   Gated SA+SWA: Y = sigmoid(gamma_sa) * Y_sa + sigmoid(gamma_swa) * Y_swa (Eq. 5), with the gate
 *         LOGITS supplied by the caller.
 *   Backward of all of the above (the paper trains through it, Sec. 4.1 / Table 3).
 * The permuted copies of Q, K, V are never materialised: rows are read through the index tensor
 * and written back through it.
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers owned by the caller, contiguous row-major, 16-byte
 *     aligned: Q, Y, dY, dQ, Y_sa, Y_swa [B,Hq,n,d]; K, V, dK, dV [B,Hkv,n,d]; LSE [B,Hq,n] float.
 *     Query head hq uses kv head hq / (Hq/Hkv).  Alignment is checked on the host: a tensor, weight or
 *     workspace pointer that is not 16-byte aligned, or an index / LSE / gate array not aligned to its
 *     element, gives SA_ERR_UNSUPPORTED before anything is launched.
 *   - Size limits (SA_ERR_SHAPE beyond): n <= 2^30, B*Hq*n < 2^31 rows; the bf16 kernels additionally need one
 *     head's rows to span less than 2 GiB (n*d*2 < 2^31, SA_ERR_UNSUPPORTED beyond).
 *   - perm: int32 [perm_B, perm_H, n]; perm[..., p] is the ORIGINAL index of the token placed at
 *     permuted slot p (the index tensor of "Q[sigma]" in Sec. 3.3; it is the inverse of the map
 *     sigma(i) = slot of token i used in Eq. 3).  perm_B in {1,B}, perm_H in {1,Hq}.  NULL means the
 *     identity.  Each slice must be a bijection of 0..n-1; otherwise results are undefined (use
 *     sa_check_perm to verify).
 *   - LSE is the natural-log sum of exp(scale * <q,k>) over the visible keys, in ORIGINAL order.
 *   - The library allocates no device memory and keeps no state; work is only enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream).  Outputs are overwritten.
 *   - Every function returns an sa_status.  Argument errors are found on the host before anything
 *     is launched; nothing aborts or throws.
 */
#ifndef SA_H
#define SA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SA_OK = 0,
  SA_ERR_NULL = 1,        /* a required pointer is NULL                       */
  SA_ERR_SHAPE = 2,       /* inconsistent or non-positive sizes               */
  SA_ERR_UNSUPPORTED = 3, /* valid request this build has no kernel for       */
  SA_ERR_WORKSPACE = 4,   /* workspace missing or smaller than required       */
  SA_ERR_BAD_PERM = 5,    /* sa_check_perm found a slice that is no bijection */
  SA_ERR_HIP = 6,         /* a HIP call or launch failed                      */
  SA_ERR_STATIC_LIMIT = 7 /* sa_decode_fwd_static: the request needs more scratch memory than
                             SA_STATIC_SCRATCH_BYTES                          */
} sa_status;

typedef enum { SA_BF16 = 0, SA_F32 = 1 } sa_dtype;

/* Window between two SLOTS s (query) and t (key) in permuted order. */
typedef enum {
  SA_WIN_SYM_CIRCULAR = 0, /* 2*min(|s-t|, n-|s-t|) < w : Sec. 3.1 / Eq. 3 / App. B (SA default) */
  SA_WIN_SYM_LINEAR = 1,   /* 2*|s-t| < w               : same without the wrap-around           */
  SA_WIN_ONE_SIDED = 2     /* 0 <= s-t <= w-1           : Sec. 3.1 footnote (causal SWA default) */
} sa_window;

typedef struct {
  int32_t B, Hq, Hkv, n, d; /* Hq % Hkv == 0; d in {64,128}                                   */
  int32_t w;                /* window size >= 1; may exceed n                                  */
  int32_t window;           /* sa_window                                                       */
  int32_t causal_orig;      /* 1: also require original index of key <= that of query (App. B) */
  int32_t dtype;            /* sa_dtype of Q,K,V,Y,dY,dQ,dK,dV                                 */
  float scale;              /* softmax scale; <= 0 selects 1/sqrt(d) (Eq. 1)                   */
  int32_t perm_B, perm_H;   /* perm is [perm_B, perm_H, n]                                     */
  int32_t gate_per_dim;     /* 0: gate logits [B,Hq,n]; 1: [B,Hq,n,d] (Eq. 5 is per dimension) */
  int32_t gate_dtype;       /* sa_dtype of the gate logits and of their gradients              */
} sa_desc;

typedef enum { SA_OP_FWD = 0, SA_OP_BWD = 1, SA_OP_GATED_FWD = 2, SA_OP_GATED_BWD = 3,
               SA_OP_CHECK_PERM = 4,
               SA_OP_GATE_PROJ_BWD = 5,        /* sa_gate_proj_bwd, both branches */
               SA_OP_GATE_PROJ_BWD_SINGLE = 6, /* sa_gate_proj_bwd, single path   */
               SA_OP_DUAL_PATH_BWD = 7,        /* sa_dual_path_bwd                */
               SA_OP_SAMPLE_PERM = 8,          /* sa_sample_perm, O(n) path       */
               SA_OP_DECODE = 9,               /* sa_decode_fwd                   */
               SA_OP_BWD_ROPE = 10             /* sa_bwd_rope                     */
} sa_op;

const char* sa_status_string(sa_status s);

/* Bytes of device workspace `op` needs for this descriptor (0 if none).  Returns 0 for an invalid
 * descriptor as well; the entry points report that case. */
size_t sa_workspace_bytes(const sa_desc* desc, int op);

/* Verifies on the device that every slice of perm is a bijection of 0..n-1.  Synchronises the
 * stream.  ws: device workspace of sa_workspace_bytes(desc, SA_OP_CHECK_PERM) bytes. */
sa_status sa_check_perm(const sa_desc* desc, const int32_t* perm, void* ws, size_t ws_bytes,
                        void* stream);

/* Alg. 1 (Sec. 3.3) with the mask of App. B:  Y = unpermute(windowed_attention(permute(Q,K,V))).
 * perm NULL = identity.  LSE may be NULL.  ws is unused (may be NULL). */
sa_status sa_fwd(const sa_desc* desc, const void* Q, const void* K, const void* V,
                 const int32_t* perm, void* Y, float* LSE, void* ws, size_t ws_bytes, void* stream);

/* Samples the permutations of one layer on the device (Sec. 3.3 and App. B: sigma ~ Uniform(S_n),
 * drawn independently per layer, fresh at every step if the caller changes `seed`).  Writes perm
 * [perm_B, perm_H, n] in the convention of this header (perm[..., p] = original index of the token at
 * slot p).  Method: sort by random key.  Slice s = pb*perm_H + ph uses the SplitMix64 sequence
 *   stream = mix(mix(seed) + G*((layer << 32) | s)),  r(p) = mix(stream + G*(p+1)),  G = 0x9E3779B97F4A7C15,
 * mix = the SplitMix64 output function; the sort key of slot p is r(p) with its low 20 bits replaced
 * by p (44 random bits, ties - probability < n^2/2^45 per slice - go to the smaller p), and perm = the
 * argsort of the keys.  Deterministic in (seed, layer, slice, n); no host round trip.  layer >= 0;
 * n <= 2^20 (SA_ERR_UNSUPPORTED beyond); at most 65535 slices.
 * ws = NULL: the rank of every key is counted against all keys, O(n^2) compares per slice, no workspace.
 * ws = sa_workspace_bytes(desc, SA_OP_SAMPLE_PERM) bytes of device memory: the keys are first spread over
 * buckets by their top bits and ranked inside their bucket, O(n) work in five small launches (taken for
 * n >= 16384, where it is the faster one); the same permutation, bit for bit. */
sa_status sa_sample_perm(const sa_desc* desc, uint64_t seed, int32_t layer, int32_t* perm, void* ws,
                         size_t ws_bytes, void* stream);

/* Measurement helper: the gather and the scatter of Alg. 1 (Sec. 3.3, the two index operations around
 * the attention) with no attention in between.  For every (b, hq, slot p), with i = perm[p]:
 *   Y[b,hq,i,:] = Q[b,hq,i,:]                                   if hq is not the first head of its KV group
 *   Y[b,hq,i,:] = Q[b,hq,i,:] + K[b,hk,i,:] + V[b,hk,i,:]       if it is   (sum in fp32, rounded once)
 * so every row of Q, K and V is read once through perm and every row of Y written once through it:
 * the bytes sa_fwd must move (without LSE), as the ceiling for rows of 2*d bytes reached through the
 * index tensor.  bf16 only (SA_ERR_UNSUPPORTED otherwise).  perm NULL = identity.  No workspace. */
sa_status sa_permuted_copy(const sa_desc* desc, const void* Q, const void* K, const void* V,
                           const int32_t* perm, void* Y, void* stream);

/* Gate projections of the dual-path layer: Eq. 6 followed by Eq. 5 (Alg. 2, "Gated Combination").
 * Per token t = (b, i) let y_x[t] in R^{dm}, dm = Hq*d, be the concatenation over heads of
 * Y_x[b,h,i,:] (feature (h,e) of a token lives at [b,h,i,e]).  Then
 *   g_x[t,:] = sigmoid(W_x y_x[t]),     Y[t,:] = g_sa * y_sa[t] + g_swa * y_swa[t]   (element-wise)
 * W_sa, W_swa: [dm, dm] row-major in the tensor dtype, row = output feature (the W_g of Eq. 6).
 * Y_swa = W_swa = NULL selects the single-path attention gate of App. B: Y = sigmoid(W_sa y_sa) * y_sa.
 * G_sa, G_swa (each may be NULL): the gate values g_x, [B,Hq,n,d] in the tensor dtype, for a backward.
 * Y may not alias Y_sa or Y_swa.  bf16 with dm a multiple of 128 only (SA_ERR_UNSUPPORTED otherwise);
 * of the descriptor only B, Hq, n, d and dtype are used.  No workspace. */
sa_status sa_gate_proj_fwd(const sa_desc* desc, const void* Y_sa, const void* Y_swa, const void* W_sa,
                           const void* W_swa, void* Y, void* G_sa, void* G_swa, void* stream);

/* Backward of sa_gate_proj_fwd.  With g_x the gate values the forward wrote (G_sa, G_swa) and dY the
 * gradient with respect to Y:
 *   dz_x = dY * y_x * g_x * (1 - g_x),   dY_x[t] = dY[t] * g_x[t] + W_x^T dz_x[t],   dW_x = sum_t dz_x[t] y_x[t]^T
 * dY_sa, dY_swa: [B,Hq,n,d]; dW_sa, dW_swa: [dm, dm] like the weights; all overwritten.  The *_swa
 * arguments are all NULL for the single path.  ws: sa_workspace_bytes(desc, SA_OP_GATE_PROJ_BWD or
 * SA_OP_GATE_PROJ_BWD_SINGLE) bytes.  dz_x is rounded to the tensor dtype before the two products;
 * dW_x is accumulated in fp32 (order of the additions not fixed) and rounded once.  Same support as
 * the forward. */
sa_status sa_gate_proj_bwd(const sa_desc* desc, const void* Y_sa, const void* Y_swa, const void* W_sa,
                           const void* W_swa, const void* G_sa, const void* G_swa, const void* dY,
                           void* dY_sa, void* dY_swa, void* dW_sa, void* dW_swa,
                           void* ws, size_t ws_bytes, void* stream);

/* App. B ("Attention" item), App. C (training setup) and Sec. 4.2: RoPE is applied to Q and K with each token's
 * ORIGINAL position, before any shuffling; RoFormer Sec. 3.2.2 defines the rotation: pair i of the row at
 * position m turns by m * base^(-2i/d).
 * sa_rope_table fills table [n][d/2][2] (device, fp32: cos then sin of (pos0 + m) * base^(-2i/d), evaluated in
 * fp64); it depends on (n, d, base, pos0) only, so a caller builds it once and keeps it.  d = 64 or 128,
 * base > 1, pos0 >= 0. */
sa_status sa_rope_table(int32_t n, int32_t d, double base, int32_t pos0, float* table, void* stream);

/* Rotates Q [B,Hq,n,d] and K [B,Hkv,n,d] (desc->dtype; either may be NULL and is then skipped) into Q_out,
 * K_out (same layout; may alias the inputs).  interleaved = 0: pair i = (x[i], x[i+d/2]) (split halves, the
 * default reading); 1: pair i = (x[2i], x[2i+1]) (as RoFormer prints it).  inverse = 1 turns by the negative
 * angle: applied to the gradients of the rotated Q, K it is the backward of this call.  `table` as written by
 * sa_rope_table for the same n and d.  The result feeds sa_fwd / sa_bwd unchanged. */
sa_status sa_rope(const sa_desc* desc, const void* Q, const void* K, const float* table, int32_t interleaved,
                  int32_t inverse, void* Q_out, void* K_out, void* stream);

/* sa_fwd with the rotation of Q fused into its load path (the prefill setting of Sec. 4.2: RoPE on original
 * positions, then stochastic attention): Q arrives UNROTATED and each query row is rotated on its original
 * position while it is staged; K arrives ROTATED (sa_rope with Q = NULL; a K row is reused by every query
 * head of its group and by several workgroups, so it is rotated once, in memory).  rope_table, interleaved: as
 * for sa_rope.  perm = NULL: identity.  bf16 only (SA_ERR_UNSUPPORTED otherwise).  No workspace. */
sa_status sa_fwd_rope(const sa_desc* desc, const void* Q, const void* K, const void* V, const int32_t* perm,
                      const float* rope_table, int32_t interleaved, void* Y, float* LSE, void* stream);

/* The backward of sa_fwd_rope (App. B "Attention" item, App. C, Sec. 4.2: RoPE on original positions, then
 * stochastic attention; the gradient of Eq. 1 over the visible set of Eq. 3 / App. B, and the transpose of the
 * rotation of RoFormer Sec. 3.2.2).  Q arrives UNROTATED and K ROTATED, as for sa_fwd_rope; Y, LSE: what
 * sa_fwd_rope returned; dY: gradient w.r.t. Y.  Each query row is rotated while the dQ kernel stages it (the
 * rotated rows, rounded to bf16 as in the forward, are kept in the workspace for the dK/dV kernel, which
 * streams them) and dQ is turned back in that kernel's epilogue: dQ is the gradient w.r.t. the UNROTATED Q.
 * dk_unrotated = 1: dK is turned back in the dK/dV kernel's epilogue as well (gradient w.r.t. the unrotated K,
 * what a caller that rotated K with sa_rope needs); 0: dK is the gradient w.r.t. the rotated K as given.
 * dV as in sa_bwd.  All of dQ, dK, dV are overwritten.  bf16 only (SA_ERR_UNSUPPORTED otherwise).
 * ws: sa_workspace_bytes(desc, SA_OP_BWD_ROPE) bytes of device memory (SA_ERR_WORKSPACE if smaller). */
sa_status sa_bwd_rope(const sa_desc* desc, const void* Q, const void* K, const void* V, const int32_t* perm,
                      const float* rope_table, int32_t interleaved, int32_t dk_unrotated, const void* Y,
                      const float* LSE, const void* dY, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
                      void* stream);

/* Alg. 2 as printed (the dual-path layer between the Q/K/V and the output projections):
 *   Y_sa = StochasticAttn(Q,K,V; perm) [sa_fwd with `sa`],  Y_swa = SWA(Q,K,V) [sa_fwd with `swa`, identity],
 *   g_x = sigmoid(Y_x W_x^T) over the model dimension (Eq. 6),  Y = g_sa * Y_sa + g_swa * Y_swa (Eq. 5).
 * Y_sa, Y_swa are required buffers [B,Hq,n,d]; G_sa, G_swa, LSE_sa, LSE_swa may be NULL at inference
 * and are what sa_dual_path_bwd needs.  Same support as sa_gate_proj_fwd.  No workspace. */
sa_status sa_dual_path_fwd(const sa_desc* sa, const sa_desc* swa, const void* Q, const void* K, const void* V,
                           const int32_t* perm, const void* W_sa, const void* W_swa, void* Y, void* Y_sa,
                           void* Y_swa, void* G_sa, void* G_swa, float* LSE_sa, float* LSE_swa, void* stream);

/* Backward of sa_dual_path_fwd: dQ, dK, dV (sums over both branches) and dW_sa, dW_swa from dY.
 * ws: sa_workspace_bytes(sa, SA_OP_DUAL_PATH_BWD) bytes. */
sa_status sa_dual_path_bwd(const sa_desc* sa, const sa_desc* swa, const void* Q, const void* K, const void* V,
                           const int32_t* perm, const void* W_sa, const void* W_swa, const void* Y_sa,
                           const void* Y_swa, const void* G_sa, const void* G_swa, const float* LSE_sa,
                           const float* LSE_swa, const void* dY, void* dQ, void* dK, void* dV, void* dW_sa,
                           void* dW_swa, void* ws, size_t ws_bytes, void* stream);

/* Decoding step of the inference setting (Sec. 4.2: the sparse modes are used for the prompt only, every
 * generated token then attends to the whole K/V cache): one query row per (b, hq), plain softmax attention
 * (Eq. 1 with every cached row visible) over rows 0..len-1 of the caches.  The caches hold K and V in the
 * original order (the permutation never leaves sa_fwd).
 * q [B,Hq,d], K, V [B,Hkv,n,d] with desc->n the capacity of the cache (the stride between heads), 1 <= len <= n
 * (SA_ERR_SHAPE otherwise), Y [B,Hq,d], LSE [B,Hq] (fp32, may be NULL); all device memory, desc->dtype.
 * desc->w, window, causal_orig and the perm and gate fields must be valid but are not used.  B*Hq <= 65535.
 * ws: sa_workspace_bytes(desc, SA_OP_DECODE) bytes (partial results of the chunks the cache is cut into; the
 * size depends on the capacity, not on len). */
sa_status sa_decode_fwd(const sa_desc* desc, const void* q, const void* K, const void* V, int32_t len, void* Y,
                        float* LSE, void* ws, size_t ws_bytes, void* stream);

/* sa_decode_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same
 * results as sa_decode_fwd, but the partial results of the chunks live in a buffer of
 * SA_STATIC_SCRATCH_BYTES that is part of the library image (one copy per GPU the library runs on, held
 * until the process ends).  The call allocates and frees nothing.
 * A descriptor whose sa_workspace_bytes(desc, SA_OP_DECODE) exceeds SA_STATIC_SCRATCH_BYTES is refused with
 * SA_ERR_STATIC_LIMIT before anything is launched (8 MiB covers, e.g., B = 1 with 32 heads of 128 over a
 * cache of 131072 rows: 4.3 MB).  The first call on a device looks the buffer's address up (no allocation;
 * make that call outside a graph capture).  All calls on one GPU share the one buffer: calls that overlap
 * on the same GPU (different streams or threads) race; calls on one stream are ordered and safe. */
#define SA_STATIC_SCRATCH_BYTES (8u << 20)
sa_status sa_decode_fwd_static(const sa_desc* desc, const void* q, const void* K, const void* V, int32_t len,
                               void* Y, float* LSE, void* stream);

/* sa_decode_fwd for a batch whose sequences have different numbers of cached rows: lens [B] (int32, device
 * memory) gives the rows of each sequence, max_len (host, 1 <= max_len <= n) an upper bound of them that sizes the
 * launch.  The values of lens cannot be checked on the host: each is clamped to 1..max_len on the device. */
sa_status sa_decode_fwd_varlen(const sa_desc* desc, const void* q, const void* K, const void* V,
                               const int32_t* lens, int32_t max_len, void* Y, float* LSE, void* ws,
                               size_t ws_bytes, void* stream);

/* Eq. 1: windowed attention in the original order (sa_fwd with the identity permutation). */
sa_status swa_fwd(const sa_desc* desc, const void* Q, const void* K, const void* V,
                  void* Y, float* LSE, void* ws, size_t ws_bytes, void* stream);

/* Alg. 2 / Eq. 5 with the gate logits as inputs.  `sa` and `swa` describe the masks of the two
 * branches and must agree in every other field.  gate_sa / gate_swa: logits, [B,Hq,n] or
 * [B,Hq,n,d] per sa->gate_per_dim, of sa->gate_dtype.
 * Y_sa, Y_swa (branch outputs, needed by the backward), LSE_sa, LSE_swa may each be NULL.
 * ws: sa_workspace_bytes(sa, SA_OP_GATED_FWD) bytes, needed only in the bf16 configuration when Y_swa is
 * NULL (the sliding-window branch's rows are kept there).  In the bf16 configuration the sum of Eq. 5 is
 * formed in fp32 from the stochastic branch's fp32 accumulators and the sliding-window branch's rows as
 * the bf16 tensor they are stored as, and rounded once. */
sa_status gated_sa_swa_fwd(const sa_desc* sa, const sa_desc* swa,
                           const void* Q, const void* K, const void* V, const int32_t* perm,
                           const void* gate_sa, const void* gate_swa,
                           void* Y, void* Y_sa, void* Y_swa, float* LSE_sa, float* LSE_swa,
                           void* ws, size_t ws_bytes, void* stream);

/* Backward of sa_fwd (swa == NULL) or of gated_sa_swa_fwd (swa != NULL).
 * Ungated: Y_sa and LSE_sa are the forward's Y and LSE; gate_*, Y_swa, LSE_swa, dgate_* are
 * ignored (may be NULL).  Gated: all of them are required.
 * dQ [B,Hq,n,d], dK, dV [B,Hkv,n,d] (summed over the query heads of a group), dgate_* like the
 * logits; all overwritten.  ws: sa_workspace_bytes(sa, SA_OP_BWD or SA_OP_GATED_BWD) bytes. */
sa_status sa_bwd(const sa_desc* sa, const sa_desc* swa,
                 const void* Q, const void* K, const void* V, const int32_t* perm,
                 const void* gate_sa, const void* gate_swa,
                 const void* Y_sa, const void* Y_swa, const float* LSE_sa, const float* LSE_swa,
                 const void* dY,
                 void* dQ, void* dK, void* dV, void* dgate_sa, void* dgate_swa,
                 void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SA_H */
