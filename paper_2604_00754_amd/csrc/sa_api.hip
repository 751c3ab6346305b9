// Host side of libsa: the extern "C" entry points declared in include/sa.h.
// Validation happens here, before any launch; kernels live in the other files of this directory.
#include <math.h>

#include <atomic>
#include <initializer_list>
#include <mutex>

#include "sa_common.h"

namespace {

using sa::Pass;
using sa::Window;

bool desc_shape_ok(const sa_desc* c) {
  if (c->B < 1 || c->Hq < 1 || c->Hkv < 1 || c->n < 1 || c->d < 1 || c->w < 1) return false;
  if (c->Hq % c->Hkv != 0) return false;
  if (c->window < SA_WIN_SYM_CIRCULAR || c->window > SA_WIN_ONE_SIDED) return false;
  if (!(c->perm_B == 1 || c->perm_B == c->B)) return false;
  if (!(c->perm_H == 1 || c->perm_H == c->Hq)) return false;
  if (c->n > (1 << 30)) return false;  // slot arithmetic is done in int32 with headroom for t in (-n, 2n)
  if ((long long)c->B * c->Hq * c->n > 0x7fffffffll) return false;  // row counts are kept in 32-bit integers
  return true;
}

sa_status validate_desc(const sa_desc* c) {
  if (!c) return SA_ERR_NULL;
  if (!desc_shape_ok(c)) return SA_ERR_SHAPE;
  if (!(c->d == 64 || c->d == 128)) return SA_ERR_UNSUPPORTED;
  if (!(c->dtype == SA_BF16 || c->dtype == SA_F32)) return SA_ERR_UNSUPPORTED;
  if (!(c->gate_dtype == SA_BF16 || c->gate_dtype == SA_F32)) return SA_ERR_UNSUPPORTED;
  if (!(c->gate_per_dim == 0 || c->gate_per_dim == 1)) return SA_ERR_SHAPE;
  if (!(c->causal_orig == 0 || c->causal_orig == 1)) return SA_ERR_SHAPE;
  if (!(c->scale == c->scale) || isinf(c->scale)) return SA_ERR_SHAPE;
  return SA_OK;
}

// Eq. 3 / App. B window as unwrapped offsets.  "2*dist < w" on integers is dist <= (w-1)/2.
Window make_window(const sa_desc* c) {
  Window win;
  const long long n = c->n, w = c->w;
  const long long h = (w - 1) / 2;
  if (c->window == SA_WIN_SYM_CIRCULAR) {
    const long long hl = h < (n - 1) / 2 ? h : (n - 1) / 2;
    const long long hr = h < n - 1 - hl ? h : n - 1 - hl;
    win.L = (int)hl;
    win.R = (int)hr;
    win.circular = 1;
  } else if (c->window == SA_WIN_SYM_LINEAR) {
    win.L = win.R = (int)(h < n - 1 ? h : n - 1);
    win.circular = 0;
  } else {
    win.L = (int)(w - 1 < n - 1 ? w - 1 : n - 1);
    win.R = 0;
    win.circular = 0;
  }
  return win;
}

Pass make_pass(const sa_desc* c, const void* Q, const void* K, const void* V, const int32_t* perm) {
  Pass p = {};
  p.Q = Q; p.K = K; p.V = V; p.perm = perm;
  p.B = c->B; p.Hq = c->Hq; p.Hkv = c->Hkv; p.n = c->n; p.d = c->d; p.g = c->Hq / c->Hkv;
  p.perm_B = perm ? c->perm_B : 1;
  p.perm_H = perm ? c->perm_H : 1;
  p.win = make_window(c);
  p.causal = c->causal_orig;
  p.scale = c->scale > 0.f ? c->scale : 1.0f / sqrtf((float)c->d);
  p.hq_only = -1;
  return p;
}

// The bf16 kernels address the rows of one head with 32-bit byte offsets.
bool head_span_ok(const sa_desc* c) {
  return c->dtype != SA_BF16 || (long long)c->n * c->d * 2 < (1ll << 31);
}

bool same_problem(const sa_desc* a, const sa_desc* b) {
  return a->B == b->B && a->Hq == b->Hq && a->Hkv == b->Hkv && a->n == b->n && a->d == b->d &&
         a->dtype == b->dtype && a->gate_per_dim == b->gate_per_dim && a->gate_dtype == b->gate_dtype;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Tensors are read and written with 16-byte vector accesses (and copied into LDS 16 bytes at a time); index,
// LSE and gate arrays with their element size.  Null pointers pass: they are optional arguments here.
// gate logits: per-dimension tensors are read like the other tensors, per-row ones element by element
size_t gate_alignment(const sa_desc* c) { return c->gate_per_dim ? 16 : (c->gate_dtype == SA_F32 ? 4 : 2); }

bool aligned_to(size_t a, std::initializer_list<const void*> ptrs) {
  for (const void* q : ptrs)
    if (q && (reinterpret_cast<uintptr_t>(q) & (a - 1))) return false;
  return true;
}

struct BwdWorkspace {
  size_t off_Da, off_Db, off_dOa, off_dOb, total;
};

BwdWorkspace bwd_workspace(const sa_desc* c, bool gated) {
  BwdWorkspace w = {};
  const size_t rows = (size_t)c->B * c->Hq * c->n;
  const size_t esize = c->dtype == SA_BF16 ? 2 : 4;
  size_t off = 0;
  w.off_Da = off; off += align256(rows * sizeof(float));
  if (gated) {
    w.off_Db = off; off += align256(rows * sizeof(float));
    w.off_dOa = off; off += align256(rows * c->d * esize);
    w.off_dOb = off; off += align256(rows * c->d * esize);
  }
  w.total = off;
  return w;
}

// sa_dual_path_bwd: gate-projection workspace | dY_sa | dY_swa | D_sa | D_swa
struct DualBwdWorkspace {
  size_t off_gp, off_dYa, off_dYb, off_Da, off_Db, total;
};

DualBwdWorkspace dual_bwd_workspace(const sa_desc* c) {
  DualBwdWorkspace w = {};
  const size_t rows = (size_t)c->B * c->Hq * c->n;
  size_t off = 0;
  w.off_gp = off; off += align256(sa::gate_proj_bwd_workspace_bytes(c->B, c->Hq, c->n, c->d, true));
  w.off_dYa = off; off += align256(rows * c->d * 2);
  w.off_dYb = off; off += align256(rows * c->d * 2);
  w.off_Da = off; off += align256(rows * sizeof(float));
  w.off_Db = off; off += align256(rows * sizeof(float));
  w.total = off;
  return w;
}

// The bf16 gated forward parks the first branch's rows (bf16, the tensor dtype) here when the caller does not
// keep them; the second branch's epilogue reads them back for the gated sum of Eq. 5.
size_t gated_fwd_workspace(const sa_desc* c) {
  if (c->dtype != SA_BF16) return 0;
  return align256((size_t)c->B * c->Hq * c->n * c->d * 2);
}

// Scratch memory of sa_decode_fwd_static: one copy per GPU the library runs on, held until the process ends.
// In host code the array's name is only a stand-in for the device symbol; the address a kernel may use is
// looked up once per device (static_scratch_ptr) and kept.
constexpr size_t kStaticScratchBytes = (size_t)SA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, or nullptr (with *err set) if it cannot be had.
void* static_scratch_ptr(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (*err != hipSuccess || !ptr) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  return ptr;
}

sa_status hip_status(hipError_t e) { return e == hipSuccess ? SA_OK : (e == hipErrorNotSupported ? SA_ERR_UNSUPPORTED : SA_ERR_HIP); }

hipError_t run_fwd(const sa_desc* c, const Pass& p, hipStream_t st) {
  return c->dtype == SA_F32 ? sa::launch_fwd_rowwise_f32(p, st) : sa::launch_fwd_mfma_bf16(p, st);
}

hipError_t run_bwd(const sa_desc* c, const Pass& p, hipStream_t st) {
  return c->dtype == SA_F32 ? sa::launch_bwd_rowwise_f32(p, st) : sa::launch_bwd_mfma_bf16(p, st);
}

}  // namespace

extern "C" {

const char* sa_status_string(sa_status s) {
  switch (s) {
    case SA_OK: return "ok";
    case SA_ERR_NULL: return "required pointer is NULL";
    case SA_ERR_SHAPE: return "invalid or inconsistent sizes";
    case SA_ERR_UNSUPPORTED: return "unsupported configuration";
    case SA_ERR_WORKSPACE: return "workspace missing or too small";
    case SA_ERR_BAD_PERM: return "perm is not a bijection of 0..n-1";
    case SA_ERR_HIP: return "HIP call failed";
    case SA_ERR_STATIC_LIMIT: return "request needs more scratch memory than the static buffer holds";
  }
  return "unknown status";
}

size_t sa_workspace_bytes(const sa_desc* c, int op) {
  if (validate_desc(c) != SA_OK) return 0;
  switch (op) {
    case SA_OP_FWD: return 0;
    case SA_OP_GATED_FWD: return gated_fwd_workspace(c);
    case SA_OP_BWD: return bwd_workspace(c, false).total;
    case SA_OP_GATED_BWD: return bwd_workspace(c, true).total;
    case SA_OP_CHECK_PERM: return align256((size_t)c->perm_B * c->perm_H * c->n * sizeof(int)) + 256;
    case SA_OP_GATE_PROJ_BWD: return sa::gate_proj_bwd_workspace_bytes(c->B, c->Hq, c->n, c->d, true);
    case SA_OP_GATE_PROJ_BWD_SINGLE: return sa::gate_proj_bwd_workspace_bytes(c->B, c->Hq, c->n, c->d, false);
    case SA_OP_DUAL_PATH_BWD: return dual_bwd_workspace(c).total;
    case SA_OP_SAMPLE_PERM: return sa::sample_perm_workspace_bytes(c->perm_B * c->perm_H, c->n);
    case SA_OP_DECODE: return align256(sa::decode_workspace_bytes(c->B, c->Hq, c->Hkv, c->n, c->d));
    case SA_OP_BWD_ROPE:  // D | the rotated Q rows
      return bwd_workspace(c, false).total + align256((size_t)c->B * c->Hq * c->n * c->d * 2);
    default: return 0;
  }
}

sa_status sa_check_perm(const sa_desc* c, const int32_t* perm, void* ws, size_t ws_bytes, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!perm) return SA_ERR_NULL;
  const size_t need = sa_workspace_bytes(c, SA_OP_CHECK_PERM);
  if (!aligned_to(4, {perm, ws})) return SA_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < need) return SA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  int* seen = reinterpret_cast<int*>(ws);
  int* flag = reinterpret_cast<int*>(reinterpret_cast<char*>(ws) + need - 256);
  hipError_t e = sa::launch_check_perm(perm, c->perm_B * c->perm_H, c->n, seen, flag, st);
  if (e != hipSuccess) return SA_ERR_HIP;
  int host_flag = 0;
  e = hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return SA_ERR_HIP;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return SA_ERR_HIP;
  return host_flag ? SA_ERR_BAD_PERM : SA_OK;
}

sa_status sa_fwd(const sa_desc* c, const void* Q, const void* K, const void* V, const int32_t* perm,
                 void* Y, float* LSE, void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!Q || !K || !V || !Y) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, Y}) || !aligned_to(4, {perm, LSE})) return SA_ERR_UNSUPPORTED;
  if (!head_span_ok(c)) return SA_ERR_UNSUPPORTED;
  Pass p = make_pass(c, Q, K, V, perm);
  p.Y = Y;
  p.LSE = LSE;
  return hip_status(run_fwd(c, p, (hipStream_t)stream));
}

namespace {
sa_status decode_common(const sa_desc* c, const void* q, const void* K, const void* V, const int32_t* lens,
                        int32_t len, void* Y, float* LSE, void* ws, size_t ws_bytes, void* stream);
}

sa_status sa_decode_fwd(const sa_desc* c, const void* q, const void* K, const void* V, int32_t len, void* Y,
                        float* LSE, void* ws, size_t ws_bytes, void* stream) {
  return decode_common(c, q, K, V, nullptr, len, Y, LSE, ws, ws_bytes, stream);
}

sa_status sa_decode_fwd_static(const sa_desc* c, const void* q, const void* K, const void* V, int32_t len, void* Y,
                               float* LSE, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  // the size is judged before the device is touched: a request that cannot fit never reaches the GPU
  const size_t need = sa_workspace_bytes(c, SA_OP_DECODE);
  if (need > kStaticScratchBytes) return SA_ERR_STATIC_LIMIT;
  if (!q || !K || !V || !Y) return SA_ERR_NULL;
  if (len < 1 || len > c->n) return SA_ERR_SHAPE;
  hipError_t e = hipSuccess;
  void* ptr = static_scratch_ptr(&e);
  if (!ptr) return SA_ERR_HIP;
  // every partial result the merge kernel reads is written by the partial kernel of the same call, so nothing
  // in the buffer has to start at zero
  return decode_common(c, q, K, V, nullptr, len, Y, LSE, ptr, kStaticScratchBytes, stream);
}

sa_status sa_decode_fwd_varlen(const sa_desc* c, const void* q, const void* K, const void* V, const int32_t* lens,
                               int32_t max_len, void* Y, float* LSE, void* ws, size_t ws_bytes, void* stream) {
  if (!lens) return SA_ERR_NULL;
  return decode_common(c, q, K, V, lens, max_len, Y, LSE, ws, ws_bytes, stream);
}

namespace {
sa_status decode_common(const sa_desc* c, const void* q, const void* K, const void* V, const int32_t* lens,
                        int32_t len, void* Y, float* LSE, void* ws, size_t ws_bytes, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!q || !K || !V || !Y) return SA_ERR_NULL;
  if (len < 1 || len > c->n) return SA_ERR_SHAPE;
  if (!aligned_to(16, {q, K, V, Y, ws}) || !aligned_to(4, {lens, LSE})) return SA_ERR_UNSUPPORTED;
  if ((long long)c->B * c->Hq > 65535) return SA_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < sa_workspace_bytes(c, SA_OP_DECODE)) return SA_ERR_WORKSPACE;
  sa::Decode d = {};
  d.q = q; d.K = K; d.V = V; d.Y = Y; d.LSE = LSE;
  d.part = reinterpret_cast<float*>(ws);
  d.B = c->B; d.Hq = c->Hq; d.Hkv = c->Hkv; d.n = c->n; d.d = c->d; d.len = len;
  d.bf16 = c->dtype == SA_BF16;
  d.scale = c->scale > 0.f ? c->scale : 1.0f / sqrtf((float)c->d);
  d.lens = lens;
  return hip_status(sa::launch_decode(d, (hipStream_t)stream));
}
}  // namespace

sa_status sa_sample_perm(const sa_desc* c, uint64_t seed, int32_t layer, int32_t* perm, void* ws, size_t ws_bytes,
                         void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!perm) return SA_ERR_NULL;
  if (layer < 0) return SA_ERR_SHAPE;
  if (!aligned_to(4, {perm})) return SA_ERR_UNSUPPORTED;
  if (c->n > (1 << 20)) return SA_ERR_UNSUPPORTED;
  const int slices = c->perm_B * c->perm_H;
  if (ws && ws_bytes < sa::sample_perm_workspace_bytes(slices, c->n)) return SA_ERR_WORKSPACE;
  return hip_status(sa::launch_sample_perm(perm, slices, c->n, seed, layer, ws, (hipStream_t)stream));
}

sa_status sa_fwd_rope(const sa_desc* c, const void* Q, const void* K, const void* V, const int32_t* perm,
                      const float* rope_table, int32_t interleaved, void* Y, float* LSE, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!Q || !K || !V || !Y || !rope_table) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, Y}) || !aligned_to(4, {perm, LSE})) return SA_ERR_UNSUPPORTED;
  if (!aligned_to(8, {rope_table})) return SA_ERR_UNSUPPORTED;
  if (!(interleaved == 0 || interleaved == 1)) return SA_ERR_SHAPE;
  if (c->dtype != SA_BF16 || !head_span_ok(c)) return SA_ERR_UNSUPPORTED;
  Pass p = make_pass(c, Q, K, V, perm);
  p.Y = Y;
  p.LSE = LSE;
  p.rope_table = rope_table;
  p.rope_interleaved = interleaved;
  return hip_status(run_fwd(c, p, (hipStream_t)stream));
}

sa_status sa_rope_table(int32_t n, int32_t d, double base, int32_t pos0, float* table, void* stream) {
  if (!table) return SA_ERR_NULL;
  if (!aligned_to(8, {table})) return SA_ERR_UNSUPPORTED;
  if (n < 1 || pos0 < 0 || (long long)n + pos0 > 0x7fffffffLL || !(base > 1.0) || isinf(base)) return SA_ERR_SHAPE;
  if (!(d == 64 || d == 128)) return SA_ERR_UNSUPPORTED;
  return hip_status(sa::launch_rope_table(table, n, d, base, pos0, (hipStream_t)stream));
}

sa_status sa_rope(const sa_desc* c, const void* Q, const void* K, const float* table, int32_t interleaved,
                  int32_t inverse, void* Q_out, void* K_out, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!table || (!Q && !K) || (Q && !Q_out) || (K && !K_out)) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, Q_out, K_out}) || !aligned_to(8, {table})) return SA_ERR_UNSUPPORTED;
  if (!(interleaved == 0 || interleaved == 1) || !(inverse == 0 || inverse == 1)) return SA_ERR_SHAPE;
  const int bf16 = c->dtype == SA_BF16;
  hipError_t e = hipSuccess;
  if (Q) e = sa::launch_rope_apply(Q, Q_out, table, c->B * c->Hq, c->n, c->d, bf16, interleaved, inverse, (hipStream_t)stream);
  if (e == hipSuccess && K)
    e = sa::launch_rope_apply(K, K_out, table, c->B * c->Hkv, c->n, c->d, bf16, interleaved, inverse, (hipStream_t)stream);
  return hip_status(e);
}

sa_status sa_permuted_copy(const sa_desc* c, const void* Q, const void* K, const void* V,
                           const int32_t* perm, void* Y, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!Q || !K || !V || !Y) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, Y}) || !aligned_to(4, {perm})) return SA_ERR_UNSUPPORTED;
  if (c->dtype != SA_BF16) return SA_ERR_UNSUPPORTED;
  Pass p = make_pass(c, Q, K, V, perm);
  p.Y = Y;
  return hip_status(sa::launch_permuted_copy_bf16(p, (hipStream_t)stream));
}

sa_status sa_gate_proj_fwd(const sa_desc* c, const void* Y_sa, const void* Y_swa, const void* W_sa,
                           const void* W_swa, void* Y, void* G_sa, void* G_swa, void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!Y_sa || !W_sa || !Y) return SA_ERR_NULL;
  if ((Y_swa == nullptr) != (W_swa == nullptr)) return SA_ERR_NULL;
  if (!aligned_to(16, {Y_sa, Y_swa, W_sa, W_swa, Y, G_sa, G_swa})) return SA_ERR_UNSUPPORTED;
  if (c->dtype != SA_BF16) return SA_ERR_UNSUPPORTED;
  if (((long)c->Hq * c->d) % 128 != 0) return SA_ERR_UNSUPPORTED;  // whole 128-feature tiles
  return hip_status(sa::launch_gate_proj_fwd_bf16(c->B, c->Hq, c->n, c->d, Y_sa, Y_swa, W_sa, W_swa, Y, G_sa,
                                                  G_swa, (hipStream_t)stream));
}

sa_status sa_gate_proj_bwd(const sa_desc* c, const void* Y_sa, const void* Y_swa, const void* W_sa,
                           const void* W_swa, const void* G_sa, const void* G_swa, const void* dY,
                           void* dY_sa, void* dY_swa, void* dW_sa, void* dW_swa, void* ws, size_t ws_bytes,
                           void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!Y_sa || !W_sa || !G_sa || !dY || !dY_sa || !dW_sa) return SA_ERR_NULL;
  const bool dual = Y_swa != nullptr;
  if (dual != (W_swa != nullptr) || dual != (G_swa != nullptr) || dual != (dY_swa != nullptr) ||
      dual != (dW_swa != nullptr))
    return SA_ERR_NULL;
  if (!aligned_to(16, {Y_sa, Y_swa, W_sa, W_swa, G_sa, G_swa, dY, dY_sa, dY_swa, dW_sa, dW_swa, ws}))
    return SA_ERR_UNSUPPORTED;
  if (c->dtype != SA_BF16) return SA_ERR_UNSUPPORTED;
  if (((long)c->Hq * c->d) % 128 != 0) return SA_ERR_UNSUPPORTED;
  const size_t need = sa::gate_proj_bwd_workspace_bytes(c->B, c->Hq, c->n, c->d, dual);
  if (!ws || ws_bytes < need) return SA_ERR_WORKSPACE;
  return hip_status(sa::launch_gate_proj_bwd_bf16(c->B, c->Hq, c->n, c->d, Y_sa, Y_swa, W_sa, W_swa, G_sa, G_swa, dY,
                                                  dY_sa, dY_swa, dW_sa, dW_swa, ws, (hipStream_t)stream));
}

sa_status sa_dual_path_fwd(const sa_desc* sa_d, const sa_desc* swa_d, const void* Q, const void* K, const void* V,
                           const int32_t* perm, const void* W_sa, const void* W_swa, void* Y, void* Y_sa,
                           void* Y_swa, void* G_sa, void* G_swa, float* LSE_sa, float* LSE_swa, void* stream) {
  sa_status s = validate_desc(sa_d);
  if (s != SA_OK) return s;
  s = validate_desc(swa_d);
  if (s != SA_OK) return s;
  if (!same_problem(sa_d, swa_d)) return SA_ERR_SHAPE;
  if (!Q || !K || !V || !W_sa || !W_swa || !Y || !Y_sa || !Y_swa) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, W_sa, W_swa, Y, Y_sa, Y_swa, G_sa, G_swa}) || !aligned_to(4, {perm, LSE_sa, LSE_swa}))
    return SA_ERR_UNSUPPORTED;
  if (sa_d->dtype != SA_BF16 || ((long)sa_d->Hq * sa_d->d) % 128 != 0) return SA_ERR_UNSUPPORTED;
  s = sa_fwd(sa_d, Q, K, V, perm, Y_sa, LSE_sa, nullptr, 0, stream);
  if (s != SA_OK) return s;
  s = sa_fwd(swa_d, Q, K, V, nullptr, Y_swa, LSE_swa, nullptr, 0, stream);
  if (s != SA_OK) return s;
  return sa_gate_proj_fwd(sa_d, Y_sa, Y_swa, W_sa, W_swa, Y, G_sa, G_swa, stream);
}

sa_status sa_dual_path_bwd(const sa_desc* sa_d, const sa_desc* swa_d, const void* Q, const void* K, const void* V,
                           const int32_t* perm, const void* W_sa, const void* W_swa, const void* Y_sa,
                           const void* Y_swa, const void* G_sa, const void* G_swa, const float* LSE_sa,
                           const float* LSE_swa, const void* dY, void* dQ, void* dK, void* dV, void* dW_sa,
                           void* dW_swa, void* ws, size_t ws_bytes, void* stream) {
  sa_status s = validate_desc(sa_d);
  if (s != SA_OK) return s;
  s = validate_desc(swa_d);
  if (s != SA_OK) return s;
  if (!same_problem(sa_d, swa_d)) return SA_ERR_SHAPE;
  if (!Q || !K || !V || !W_sa || !W_swa || !Y_sa || !Y_swa || !G_sa || !G_swa || !LSE_sa || !LSE_swa || !dY ||
      !dQ || !dK || !dV || !dW_sa || !dW_swa)
    return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, W_sa, W_swa, Y_sa, Y_swa, G_sa, G_swa, dY, dQ, dK, dV, dW_sa, dW_swa, ws}) ||
      !aligned_to(4, {perm, LSE_sa, LSE_swa}))
    return SA_ERR_UNSUPPORTED;
  if (sa_d->dtype != SA_BF16 || ((long)sa_d->Hq * sa_d->d) % 128 != 0 || !head_span_ok(sa_d)) return SA_ERR_UNSUPPORTED;
  const DualBwdWorkspace w = dual_bwd_workspace(sa_d);
  if (!ws || ws_bytes < w.total) return SA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* base = reinterpret_cast<char*>(ws);
  void* dYa = base + w.off_dYa;
  void* dYb = base + w.off_dYb;
  // Eq. 5 / Eq. 6 backwards: gradients of the two branch outputs and of the gate weights
  hipError_t e = sa::launch_gate_proj_bwd_bf16(sa_d->B, sa_d->Hq, sa_d->n, sa_d->d, Y_sa, Y_swa, W_sa, W_swa, G_sa, G_swa,
                                               dY, dYa, dYb, dW_sa, dW_swa, base + w.off_gp, st);
  if (e != hipSuccess) return hip_status(e);
  // each attention branch on its own gradient; the second adds to the first
  const void* dO[2] = {dYb, dYa};
  const void* Yx[2] = {Y_swa, Y_sa};
  const float* lse[2] = {LSE_swa, LSE_sa};
  float* D[2] = {reinterpret_cast<float*>(base + w.off_Db), reinterpret_cast<float*>(base + w.off_Da)};
  const sa_desc* dsc[2] = {swa_d, sa_d};
  for (int x = 0; x < 2; ++x) {
    Pass p = make_pass(dsc[x], Q, K, V, x == 0 ? nullptr : perm);
    p.dO = dO[x]; p.lse_in = lse[x];
    p.O_rows = Yx[x]; p.Dsum_out = D[x];  // the dQ kernel forms rowsum(dO o O) from the rows it holds
    p.dQ = dQ; p.dK = dK; p.dV = dV; p.accumulate = x;
    e = run_bwd(dsc[x], p, st);
    if (e != hipSuccess) return hip_status(e);
  }
  return SA_OK;
}

sa_status swa_fwd(const sa_desc* c, const void* Q, const void* K, const void* V, void* Y, float* LSE,
                  void* ws, size_t ws_bytes, void* stream) {
  return sa_fwd(c, Q, K, V, nullptr, Y, LSE, ws, ws_bytes, stream);
}

sa_status gated_sa_swa_fwd(const sa_desc* sa_d, const sa_desc* swa_d, const void* Q, const void* K,
                           const void* V, const int32_t* perm, const void* gate_sa,
                           const void* gate_swa, void* Y, void* Y_sa, void* Y_swa, float* LSE_sa,
                           float* LSE_swa, void* ws, size_t ws_bytes, void* stream) {
  sa_status s = validate_desc(sa_d);
  if (s != SA_OK) return s;
  s = validate_desc(swa_d);
  if (s != SA_OK) return s;
  if (!same_problem(sa_d, swa_d)) return SA_ERR_SHAPE;
  if (!Q || !K || !V || !Y || !gate_sa || !gate_swa) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, Y, Y_sa, Y_swa, ws}) || !aligned_to(4, {perm, LSE_sa, LSE_swa}) ||
      !aligned_to(gate_alignment(sa_d), {gate_sa, gate_swa}))
    return SA_ERR_UNSUPPORTED;
  if (!head_span_ok(sa_d)) return SA_ERR_UNSUPPORTED;
  const bool bf16 = sa_d->dtype == SA_BF16;
  const size_t need = gated_fwd_workspace(sa_d);
  if (bf16 && !Y_swa && (!ws || ws_bytes < need)) return SA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;

  // sliding-window branch first (Alg. 2).  Its rows go to Y_swa if the caller keeps them, else to the
  // workspace (bf16) or to Y itself (fp32: the second pass reads a row before it overwrites it).
  Pass a = make_pass(swa_d, Q, K, V, nullptr);
  a.Y = Y_swa ? Y_swa : (bf16 ? ws : Y);
  a.LSE = LSE_swa;
  hipError_t e = run_fwd(swa_d, a, st);
  if (e != hipSuccess) return hip_status(e);

  // stochastic branch; its epilogue reads the other branch's row and forms the gated sum (Eq. 5)
  Pass b = make_pass(sa_d, Q, K, V, perm);
  b.Y = Y_sa;
  b.LSE = LSE_sa;
  b.gate_mode = 1;
  b.gate_per_dim = sa_d->gate_per_dim;
  b.gate_f32 = sa_d->gate_dtype == SA_F32;
  b.gate_this = gate_sa;
  b.gate_other = gate_swa;
  b.Y_other = a.Y;
  b.Yout = Y;
  return hip_status(run_fwd(sa_d, b, st));
}

sa_status sa_bwd(const sa_desc* sa_d, const sa_desc* swa_d, const void* Q, const void* K, const void* V,
                 const int32_t* perm, const void* gate_sa, const void* gate_swa, const void* Y_sa,
                 const void* Y_swa, const float* LSE_sa, const float* LSE_swa, const void* dY,
                 void* dQ, void* dK, void* dV, void* dgate_sa, void* dgate_swa, void* ws,
                 size_t ws_bytes, void* stream) {
  sa_status s = validate_desc(sa_d);
  if (s != SA_OK) return s;
  const bool gated = swa_d != nullptr;
  if (gated) {
    s = validate_desc(swa_d);
    if (s != SA_OK) return s;
    if (!same_problem(sa_d, swa_d)) return SA_ERR_SHAPE;
  }
  if (!Q || !K || !V || !Y_sa || !LSE_sa || !dY || !dQ || !dK || !dV) return SA_ERR_NULL;
  if (gated && (!gate_sa || !gate_swa || !Y_swa || !LSE_swa || !dgate_sa || !dgate_swa)) return SA_ERR_NULL;
  if (!aligned_to(16, {Q, K, V, Y_sa, Y_swa, dY, dQ, dK, dV, ws}) || !aligned_to(4, {perm, LSE_sa, LSE_swa}) ||
      (gated && !aligned_to(gate_alignment(sa_d), {gate_sa, gate_swa, dgate_sa, dgate_swa})))
    return SA_ERR_UNSUPPORTED;
  if (!head_span_ok(sa_d)) return SA_ERR_UNSUPPORTED;
  const BwdWorkspace w = bwd_workspace(sa_d, gated);
  if (!ws || ws_bytes < w.total) return SA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* base = reinterpret_cast<char*>(ws);

  sa::Prep pr = {};
  pr.rows = sa_d->B * sa_d->Hq * sa_d->n;
  pr.d = sa_d->d;
  pr.bf16 = sa_d->dtype == SA_BF16;
  pr.gated = gated;
  pr.gate_per_dim = sa_d->gate_per_dim;
  pr.gate_f32 = sa_d->gate_dtype == SA_F32;
  pr.dY = dY;
  pr.Y_a = Y_sa; pr.Y_b = Y_swa;
  pr.gate_a = gate_sa; pr.gate_b = gate_swa;
  pr.D_a = reinterpret_cast<float*>(base + w.off_Da);
  pr.D_b = gated ? reinterpret_cast<float*>(base + w.off_Db) : nullptr;
  pr.dO_a = gated ? base + w.off_dOa : nullptr;
  pr.dO_b = gated ? base + w.off_dOb : nullptr;
  pr.dgate_a = dgate_sa; pr.dgate_b = dgate_swa;
  // bf16, one gate per (head, token): the gate goes into the per-row scalars, both branches run on dY itself
  // (the two shifted LSE vectors take the place of the first branch gradient in the workspace)
  const bool fold = gated && !sa_d->gate_per_dim && sa_d->dtype == SA_BF16;
  pr.fold = fold;
  pr.lse_a = LSE_sa; pr.lse_b = LSE_swa;
  pr.L_a = fold ? reinterpret_cast<float*>(base + w.off_dOa) : nullptr;
  pr.L_b = fold ? pr.L_a + (size_t)pr.rows : nullptr;
  // ungated bf16: no separate pass, the dQ kernel forms rowsum(dY o Y) from the rows it holds
  const bool rowsum_in_dq = !gated && sa_d->dtype == SA_BF16;
  hipError_t e = rowsum_in_dq ? hipSuccess : sa::launch_bwd_prepare(pr, st);
  if (e != hipSuccess) return hip_status(e);

  if (gated) {
    Pass a = make_pass(swa_d, Q, K, V, nullptr);
    a.dO = fold ? dY : pr.dO_b;
    a.lse_in = fold ? pr.L_b : LSE_swa;
    a.Dsum = pr.D_b;
    a.dQ = dQ; a.dK = dK; a.dV = dV; a.accumulate = 0;
    e = run_bwd(swa_d, a, st);
    if (e != hipSuccess) return hip_status(e);
  }
  Pass b = make_pass(sa_d, Q, K, V, perm);
  b.dO = gated && !fold ? pr.dO_a : dY;
  b.lse_in = fold ? pr.L_a : LSE_sa;
  b.Dsum = pr.D_a;
  if (rowsum_in_dq) { b.O_rows = Y_sa; b.Dsum_out = pr.D_a; }
  b.dQ = dQ; b.dK = dK; b.dV = dV; b.accumulate = gated ? 1 : 0;
  return hip_status(run_bwd(sa_d, b, st));
}

sa_status sa_bwd_rope(const sa_desc* c, const void* Q, const void* K, const void* V, const int32_t* perm,
                      const float* rope_table, int32_t interleaved, int32_t dk_unrotated, const void* Y,
                      const float* LSE, const void* dY, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
                      void* stream) {
  sa_status s = validate_desc(c);
  if (s != SA_OK) return s;
  if (!Q || !K || !V || !Y || !LSE || !dY || !dQ || !dK || !dV || !rope_table) return SA_ERR_NULL;
  if ((interleaved != 0 && interleaved != 1) || (dk_unrotated != 0 && dk_unrotated != 1)) return SA_ERR_SHAPE;
  if (c->dtype != SA_BF16) return SA_ERR_UNSUPPORTED;
  if (!aligned_to(16, {Q, K, V, Y, dY, dQ, dK, dV, ws}) || !aligned_to(4, {perm, LSE}) || !aligned_to(8, {rope_table}))
    return SA_ERR_UNSUPPORTED;
  if (!head_span_ok(c)) return SA_ERR_UNSUPPORTED;
  const BwdWorkspace w = bwd_workspace(c, false);
  if (!ws || ws_bytes < sa_workspace_bytes(c, SA_OP_BWD_ROPE)) return SA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* base = reinterpret_cast<char*>(ws);

  Pass b = make_pass(c, Q, K, V, perm);
  b.rope_table = rope_table;
  b.rope_interleaved = interleaved;
  b.rope_dk = dk_unrotated;
  b.Q_rot = base + w.total;
  b.dO = dY;
  b.lse_in = LSE;
  b.O_rows = Y;  // the dQ kernel forms rowsum(dY o Y) from the rows it holds
  b.Dsum_out = reinterpret_cast<float*>(base + w.off_Da);
  b.dQ = dQ; b.dK = dK; b.dV = dV; b.accumulate = 0;
  return hip_status(sa::launch_bwd_mfma_bf16(b, st));
}

}  // extern "C"
