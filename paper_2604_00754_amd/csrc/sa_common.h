// Internal declarations shared by the host entry points and the gfx950 kernels of libsa.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sa.h"

namespace sa {

// Window of Eq. 3 / App. B rewritten on UNWRAPPED slot offsets: key slot t is inside the window of
// query slot s iff -L <= t - s <= R, where for the circular kind t runs over s-L .. s+R and is
// reduced mod n (L + R + 1 <= n, so each slot is met once), and for the other kinds 0 <= t < n.
struct Window {
  int L, R, circular;
};

// Everything one attention pass (forward or backward, one branch) needs.
struct Pass {
  const void* Q;
  const void* K;
  const void* V;
  const int32_t* perm;  // nullptr = identity
  int B, Hq, Hkv, n, d, g;
  int perm_B, perm_H;
  Window win;
  int causal;
  float scale;          // softmax scale (Eq. 1)
  // bf16 only: rotate the Q rows on their original positions while they are staged (RoPE table [n][d/2][2]
  // of sa_rope_table; nullptr = Q arrives rotated).  K always arrives rotated.  In the backward the dQ kernel
  // does the same, leaves the rotated rows in Q_rot for the dK/dV kernel (which streams them) and turns dQ back
  // in its epilogue; rope_dk: the dK/dV kernel turns dK back as well (gradient w.r.t. the unrotated K).
  const float* rope_table;
  int rope_interleaved;
  void* Q_rot;
  int rope_dk;
  // forward outputs
  void* Y;              // branch output rows, may be nullptr when only the gated sum is wanted
  float* LSE;           // may be nullptr
  // gated epilogue (Eq. 5), used by the second branch of the gated forward
  int gate_mode;        // 0 none; 1 combine: Yout = sig(ga)*this + sig(gb)*other
  int gate_per_dim, gate_f32;
  const void* gate_this;
  const void* gate_other;
  const void* Y_other;  // the other branch's rows [B,Hq,n,d] in the tensor dtype (fp32 path: may alias Yout)
  void* Yout;           // gated sum
  // backward
  const void* dO;       // gradient w.r.t. this branch's output [B,Hq,n,d]
  const float* lse_in;  // [B,Hq,n]
  const float* Dsum;    // rowsum(dO * O) [B,Hq,n]
  const void* O_rows;   // bf16 path, optional: this branch's output rows [B,Hq,n,d]; when given, the dQ kernel forms
  float* Dsum_out;      // rowsum(dO * O) itself from its stationary rows and leaves it here for the dK/dV kernel
  void* dQ;
  void* dK;
  void* dV;
  int accumulate;       // 1: add to what dQ/dK/dV already hold (second branch of the gated backward)
  int hq_only;          // >= 0: dK/dV pass restricted to this query head of every group
};

__host__ __device__ inline int perm_slice_index(int perm_B, int perm_H, int b, int hq) {
  return (perm_B == 1 ? 0 : b) * perm_H + (perm_H == 1 ? 0 : hq);
}

// kernels (each file checks its own launch geometry against the Pass on the host)
hipError_t launch_fwd_rowwise_f32(const Pass& p, hipStream_t st);
hipError_t launch_bwd_rowwise_f32(const Pass& p, hipStream_t st);
hipError_t launch_fwd_mfma_bf16(const Pass& p, hipStream_t st);
hipError_t launch_bwd_mfma_bf16(const Pass& p, hipStream_t st);

hipError_t launch_permuted_copy_bf16(const Pass& p, hipStream_t st);
// ws = nullptr: O(n^2) rank counting, no workspace; otherwise sample_perm_workspace_bytes(slices, n) bytes
hipError_t launch_sample_perm(int32_t* perm, int slices, int n, uint64_t seed, int layer, void* ws, hipStream_t st);
size_t sample_perm_workspace_bytes(int slices, int n);
// Eq. 6 + Eq. 5 (sa_gate_proj.hip); Y_swa = W_swa = nullptr selects the single-path gate
hipError_t launch_gate_proj_fwd_bf16(int B, int Hq, int n, int d, const void* Y_sa, const void* Y_swa,
                                     const void* W_sa, const void* W_swa, void* Y, void* G_sa, void* G_swa,
                                     hipStream_t st);

size_t gate_proj_bwd_workspace_bytes(int B, int Hq, int n, int d, bool dual);
hipError_t launch_gate_proj_bwd_bf16(int B, int Hq, int n, int d, const void* Y_sa, const void* Y_swa,
                                     const void* W_sa, const void* W_swa, const void* G_sa, const void* G_swa,
                                     const void* dY, void* dY_sa, void* dY_swa, void* dW_sa, void* dW_swa,
                                     void* ws, hipStream_t st);

// sa_rope.hip: (cos, sin) table [n][d/2][2] and the rotation of X [heads][n][d] (in place allowed)
hipError_t launch_rope_table(float* table, int n, int d, double base, int pos0, hipStream_t st);
hipError_t launch_rope_apply(const void* X, void* Xout, const float* table, int heads, int n, int d, int bf16,
                             int interleaved, int inverse, hipStream_t st);

// sa_decode.hip: one query row per (b, hq) over rows 0..len-1 of the K/V caches (Sec. 4.2, decoding)
struct Decode {
  const void* q;   // [B,Hq,d]
  const void* K;   // [B,Hkv,n,d], n = capacity
  const void* V;
  void* Y;         // [B,Hq,d]
  float* LSE;      // [B,Hq], may be nullptr
  float* part;     // decode_workspace_bytes(...) bytes
  const int32_t* lens;   // [B] device, or nullptr: every sequence has `len` rows; else len = the largest
  int B, Hq, Hkv, n, d, len, bf16;
  float scale;
};
size_t decode_workspace_bytes(int B, int Hq, int Hkv, int n, int d);
hipError_t launch_decode(const Decode& d, hipStream_t st);

// helpers in sa_misc.hip
hipError_t launch_check_perm(const int32_t* perm, int slices, int n, int* seen, int* flag,
                             hipStream_t st);
// D = rowsum(dO * O); for the gated case also dO_x = sig(gamma_x) * dY and the gate-logit gradients.
struct Prep {
  int rows, d;               // rows = B*Hq*n
  int bf16;                  // dtype of Y, dY, dO
  int gated, gate_per_dim, gate_f32;
  const void* dY;
  const void* Y_a;  const void* Y_b;          // branch outputs (b unused when not gated)
  const void* gate_a; const void* gate_b;
  void* dO_a; void* dO_b;                      // gated only
  float* D_a; float* D_b;
  void* dgate_a; void* dgate_b;
  // gated with one gate per (head, token) and fold != 0: the gate is folded into the per-row scalars instead
  // of into a copy of dY.  With g = sigmoid(gamma_x): dO_x = g dY, so P^T dO_x = (g P)^T dY and
  // dS_x = P (dO_x V^T - D_x) = (g P) (dY V^T - E_x) with E_x = rowsum(dY * Y_x) = D_x / g.  The backward
  // kernels then run on dY itself with LSE_x - ln g in place of LSE_x (which turns P into g P) and E_x in
  // place of D_x; g = 0 gives +inf and P = 0.  D_a / D_b receive E_x, L_a / L_b the shifted LSE.
  int fold;
  const float* lse_a; const float* lse_b;
  float* L_a; float* L_b;
};
hipError_t launch_bwd_prepare(const Prep& p, hipStream_t st);
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st);

}  // namespace sa
