// fp32 path of libsa: one wavefront per row, plain FMA arithmetic, no matrix cores.
//
// These kernels serve dtype == SA_F32 (tolerance 1e-5 against the fp64 definition).  They follow
// Alg. 1 with the permutation folded into the addressing: a wave owns one permuted slot, walks
// the slots of its window (Eq. 3), reads K/V rows through the index tensor, applies the causal
// test on original positions (Sec. 3.3, App. B), keeps an online softmax (Eq. 1) and writes the
// result to the row's original position.
#include "sa_common.h"
#include "sa_device.h"

namespace sa {
namespace {

constexpr int kWaves = 4;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const float* __restrict__ row, int d) {
  float acc = 0.f;
  for (int k = 0; k < d; k += 4) {
    f32x4 r = *reinterpret_cast<const f32x4*>(row + k);
    acc = fmaf(a_lds[k], r[0], acc);
    acc = fmaf(a_lds[k + 1], r[1], acc);
    acc = fmaf(a_lds[k + 2], r[2], acc);
    acc = fmaf(a_lds[k + 3], r[3], acc);
  }
  return acc;
}

struct RowCtx {
  bool valid;
  int b, hq, hk, s;
  const int32_t* perm;
};

__device__ __forceinline__ RowCtx decode_row(const Pass& p, long row) {
  RowCtx c;
  long total = (long)p.B * p.Hq * p.n;
  c.valid = row < total;
  if (!c.valid) row = 0;
  c.s = (int)(row % p.n);
  c.hq = (int)((row / p.n) % p.Hq);
  c.b = (int)(row / ((long)p.n * p.Hq));
  c.hk = c.hq / p.g;
  c.perm = p.perm ? p.perm + (size_t)perm_slice_index(p.perm_B, p.perm_H, c.b, c.hq) * p.n : nullptr;
  return c;
}

// Unwrapped range of the other side's slots for slot s: [s - lo_reach, s + hi_reach].
__device__ __forceinline__ void slot_range(const Pass& p, int s, int lo_reach, int hi_reach, int& t_lo, int& t_hi) {
  t_lo = s - lo_reach;
  t_hi = s + hi_reach;
  if (!p.win.circular) {
    t_lo = max(t_lo, 0);
    t_hi = min(t_hi, p.n - 1);
  }
}

__global__ __launch_bounds__(kWaves * 64) void fwd_rowwise_f32_kernel(Pass p) {
  __shared__ float qs[kWaves][128];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const RowCtx c = decode_row(p, (long)blockIdx.x * kWaves + wave);
  const int d = p.d, n = p.n;
  const int i = slot_to_orig(c.perm, c.s);
  const float* Q = reinterpret_cast<const float*>(p.Q) + (((size_t)c.b * p.Hq + c.hq) * n + i) * d;
  const float* Kh = reinterpret_cast<const float*>(p.K) + ((size_t)c.b * p.Hkv + c.hk) * n * (size_t)d;
  const float* Vh = reinterpret_cast<const float*>(p.V) + ((size_t)c.b * p.Hkv + c.hk) * n * (size_t)d;
  for (int k = lane; k < d; k += 64) qs[wave][k] = Q[k];
  __syncthreads();
  if (!c.valid) return;

  int t_lo, t_hi;
  slot_range(p, c.s, p.win.L, p.win.R, t_lo, t_hi);
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int t0 = t_lo; t0 <= t_hi; t0 += 64) {
    const int t = t0 + lane;
    const int cnt = min(64, t_hi - t0 + 1);
    int j = 0;
    bool keep = t <= t_hi;
    if (keep) {
      j = slot_to_orig(c.perm, wrap_slot(t, n));
      keep = !p.causal || j <= i;
    }
    float z = -INFINITY;
    if (keep) z = p.scale * dot_row(qs[wave], Kh + (size_t)j * d, d);
    const float m_new = fmaxf(m, wave_max(z));
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float pe = keep ? expf(z - m_safe) : 0.f;
    const float alpha = expf(m - m_safe);
    l = l * alpha + wave_sum(pe);
    o0 *= alpha;
    o1 *= alpha;
    for (int u = 0; u < cnt; ++u) {
      const float pu = __shfl(pe, u);
      const int ju = __shfl(j, u);
      if (pu != 0.f) {
        const float* v = Vh + (size_t)ju * d;
        o0 = fmaf(pu, v[lane], o0);
        if (d > 64) o1 = fmaf(pu, v[lane + 64], o1);
      }
    }
    m = m_new;
  }
  const float inv_l = 1.f / l;
  const size_t row_i = ((size_t)c.b * p.Hq + c.hq) * n + i;
  float y0 = o0 * inv_l, y1 = o1 * inv_l;
  if (p.Y) {
    float* Y = reinterpret_cast<float*>(p.Y) + row_i * d;
    Y[lane] = y0;
    if (d > 64) Y[lane + 64] = y1;
  }
  if (p.LSE && lane == 0) p.LSE[row_i] = m + logf(l);
  if (p.gate_mode) {
    // Eq. 5: independent sigmoid gates on the two branches
    const float* other = reinterpret_cast<const float*>(p.Y_other) + row_i * d;
    float* out = reinterpret_cast<float*>(p.Yout) + row_i * d;
    for (int h = 0; h < (d > 64 ? 2 : 1); ++h) {
      const int k = lane + 64 * h;
      const size_t gi = p.gate_per_dim ? row_i * d + k : row_i;
      const float ga = sigmoidf_exact(load_gate(p.gate_this, gi, p.gate_f32));
      const float gb = sigmoidf_exact(load_gate(p.gate_other, gi, p.gate_f32));
      out[k] = ga * (h ? y1 : y0) + gb * other[k];
    }
  }
}

// dQ_i = scale * sum_j dS_ij K_j with dS_ij = P_ij (<dO_i, V_j> - D_i), P_ij = exp(z_ij - LSE_i).
__global__ __launch_bounds__(kWaves * 64) void bwd_dq_rowwise_f32_kernel(Pass p) {
  __shared__ float qs[kWaves][128];
  __shared__ float gs[kWaves][128];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const RowCtx c = decode_row(p, (long)blockIdx.x * kWaves + wave);
  const int d = p.d, n = p.n;
  const int i = slot_to_orig(c.perm, c.s);
  const size_t row_i = ((size_t)c.b * p.Hq + c.hq) * n + i;
  const float* Q = reinterpret_cast<const float*>(p.Q) + row_i * d;
  const float* dO = reinterpret_cast<const float*>(p.dO) + row_i * d;
  const float* Kh = reinterpret_cast<const float*>(p.K) + ((size_t)c.b * p.Hkv + c.hk) * n * (size_t)d;
  const float* Vh = reinterpret_cast<const float*>(p.V) + ((size_t)c.b * p.Hkv + c.hk) * n * (size_t)d;
  for (int k = lane; k < d; k += 64) {
    qs[wave][k] = Q[k];
    gs[wave][k] = dO[k];
  }
  __syncthreads();
  if (!c.valid) return;
  const float lse = p.lse_in[row_i], Dv = p.Dsum[row_i];
  int t_lo, t_hi;
  slot_range(p, c.s, p.win.L, p.win.R, t_lo, t_hi);
  float a0 = 0.f, a1 = 0.f;
  for (int t0 = t_lo; t0 <= t_hi; t0 += 64) {
    const int t = t0 + lane;
    const int cnt = min(64, t_hi - t0 + 1);
    int j = 0;
    bool keep = t <= t_hi;
    if (keep) {
      j = slot_to_orig(c.perm, wrap_slot(t, n));
      keep = !p.causal || j <= i;
    }
    float dS = 0.f;
    if (keep) {
      const float z = p.scale * dot_row(qs[wave], Kh + (size_t)j * d, d);
      const float pr = expf(z - lse);
      dS = pr * (dot_row(gs[wave], Vh + (size_t)j * d, d) - Dv);
    }
    for (int u = 0; u < cnt; ++u) {
      const float su = __shfl(dS, u);
      const int ju = __shfl(j, u);
      if (su != 0.f) {
        const float* kr = Kh + (size_t)ju * d;
        a0 = fmaf(su, kr[lane], a0);
        if (d > 64) a1 = fmaf(su, kr[lane + 64], a1);
      }
    }
  }
  float* dQ = reinterpret_cast<float*>(p.dQ) + row_i * d;
  a0 *= p.scale;
  a1 *= p.scale;
  if (p.accumulate) {
    a0 += dQ[lane];
    if (d > 64) a1 += dQ[lane + 64];
  }
  dQ[lane] = a0;
  if (d > 64) dQ[lane + 64] = a1;
}

// One wave per (query head, key slot): dV_j = sum_i P_ij dO_i, dK_j = scale * sum_i dS_ij Q_i over the
// queries whose window holds this key.  With grouped heads the g partial rows are added atomically.
__global__ __launch_bounds__(kWaves * 64) void bwd_dkv_rowwise_f32_kernel(Pass p) {
  __shared__ float ks[kWaves][128];
  __shared__ float vs[kWaves][128];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const RowCtx c = decode_row(p, (long)blockIdx.x * kWaves + wave);
  const int d = p.d, n = p.n;
  const int j = slot_to_orig(c.perm, c.s);
  const size_t row_j = ((size_t)c.b * p.Hkv + c.hk) * n + j;
  const float* Kr = reinterpret_cast<const float*>(p.K) + row_j * d;
  const float* Vr = reinterpret_cast<const float*>(p.V) + row_j * d;
  const size_t qbase = ((size_t)c.b * p.Hq + c.hq) * n;
  const float* Qh = reinterpret_cast<const float*>(p.Q) + qbase * d;
  const float* dOh = reinterpret_cast<const float*>(p.dO) + qbase * d;
  for (int k = lane; k < d; k += 64) {
    ks[wave][k] = Kr[k];
    vs[wave][k] = Vr[k];
  }
  __syncthreads();
  if (!c.valid) return;
  // queries at slots s with -L <= t - s <= R, i.e. s in [t - R, t + L]
  int s_lo, s_hi;
  slot_range(p, c.s, p.win.R, p.win.L, s_lo, s_hi);
  float dv0 = 0.f, dv1 = 0.f, dk0 = 0.f, dk1 = 0.f;
  for (int s0 = s_lo; s0 <= s_hi; s0 += 64) {
    const int s = s0 + lane;
    const int cnt = min(64, s_hi - s0 + 1);
    int i = 0;
    bool keep = s <= s_hi;
    if (keep) {
      i = slot_to_orig(c.perm, wrap_slot(s, n));
      keep = !p.causal || j <= i;
    }
    float pr = 0.f, dS = 0.f;
    if (keep) {
      const float z = p.scale * dot_row(ks[wave], Qh + (size_t)i * d, d);
      pr = expf(z - p.lse_in[qbase + i]);
      dS = pr * (dot_row(vs[wave], dOh + (size_t)i * d, d) - p.Dsum[qbase + i]);
    }
    for (int u = 0; u < cnt; ++u) {
      const float pu = __shfl(pr, u);
      const float su = __shfl(dS, u);
      const int iu = __shfl(i, u);
      if (pu != 0.f) {
        const float* go = dOh + (size_t)iu * d;
        const float* qr = Qh + (size_t)iu * d;
        dv0 = fmaf(pu, go[lane], dv0);
        dk0 = fmaf(su, qr[lane], dk0);
        if (d > 64) {
          dv1 = fmaf(pu, go[lane + 64], dv1);
          dk1 = fmaf(su, qr[lane + 64], dk1);
        }
      }
    }
  }
  dk0 *= p.scale;
  dk1 *= p.scale;
  float* dK = reinterpret_cast<float*>(p.dK) + row_j * d;
  float* dV = reinterpret_cast<float*>(p.dV) + row_j * d;
  if (p.g > 1) {  // host zero-filled (or left the first branch's sums in) dK/dV
    atomicAdd(dK + lane, dk0);
    atomicAdd(dV + lane, dv0);
    if (d > 64) {
      atomicAdd(dK + lane + 64, dk1);
      atomicAdd(dV + lane + 64, dv1);
    }
  } else {
    if (p.accumulate) {
      dk0 += dK[lane];
      dv0 += dV[lane];
      if (d > 64) {
        dk1 += dK[lane + 64];
        dv1 += dV[lane + 64];
      }
    }
    dK[lane] = dk0;
    dV[lane] = dv0;
    if (d > 64) {
      dK[lane + 64] = dk1;
      dV[lane + 64] = dv1;
    }
  }
}

bool rowwise_shape_ok(const Pass& p) {
  return (p.d == 64 || p.d == 128) && p.n >= 1 && p.B >= 1 && p.Hq >= 1 && p.g >= 1 &&
         p.win.L >= 0 && p.win.R >= 0 && p.win.L < p.n && p.win.R < p.n &&
         (!p.win.circular || p.win.L + p.win.R + 1 <= p.n);
}

unsigned rowwise_blocks(const Pass& p) {
  long rows = (long)p.B * p.Hq * p.n;
  return (unsigned)((rows + kWaves - 1) / kWaves);
}

}  // namespace

hipError_t launch_fwd_rowwise_f32(const Pass& p, hipStream_t st) {
  if (!rowwise_shape_ok(p)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fwd_rowwise_f32_kernel, dim3(rowwise_blocks(p)), dim3(kWaves * 64), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_bwd_rowwise_f32(const Pass& p, hipStream_t st) {
  if (!rowwise_shape_ok(p)) return hipErrorInvalidValue;
  if (p.g > 1 && !p.accumulate) {
    const size_t bytes = (size_t)p.B * p.Hkv * p.n * p.d * sizeof(float);
    hipError_t e = launch_fill_zero(p.dK, bytes, st);
    if (e != hipSuccess) return e;
    e = launch_fill_zero(p.dV, bytes, st);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(bwd_dq_rowwise_f32_kernel, dim3(rowwise_blocks(p)), dim3(kWaves * 64), 0, st, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dkv_rowwise_f32_kernel, dim3(rowwise_blocks(p)), dim3(kWaves * 64), 0, st, p);
  return hipGetLastError();
}

}  // namespace sa
