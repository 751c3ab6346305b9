// Rotary position embeddings on ORIGINAL token positions (App. B, "Attention" item; App. C, training
// paragraph; Sec. 4.2): Q and K are rotated with the position each token has in the sequence before
// any shuffling, so the permutation never enters here.  RoFormer Sec. 3.2.2: pair i of the row at
// position m turns by m * base^(-2i/d).
//
// Two kernels.  The table kernel evaluates (cos, sin) of every (position, pair) once, in fp64 (the
// angle reaches 10^5 rad at long prefill, beyond what an fp32 product resolves), and stores them as
// fp32.  The apply kernel streams rows: one thread owns the same 8 pairs of one position for several
// heads, keeps their 16 table values in registers, and reads / writes 2 x 16 B (bf16) per head.
// HBM-bound: 2 * sizeof(T) bytes per element, the table stays in cache.
#include "sa_common.h"
#include "sa_device.h"

namespace sa {
namespace {

constexpr int ROPE_THREADS = 256;
constexpr int ROPE_HEADS_PER_BLOCK = 4;

__global__ __launch_bounds__(ROPE_THREADS) void rope_table_kernel(float2* __restrict__ table, int n, int half,
                                                                   double base, int pos0) {
  const long i = (long)blockIdx.x * ROPE_THREADS + threadIdx.x;
  if (i >= (long)n * half) return;
  const int m = (int)(i / half), pair = (int)(i % half);
  const double theta = pow(base, -(double)pair / (double)half);  // base^(-2 pair / d)
  double s, c;
  sincos((double)(pos0 + m) * theta, &s, &c);
  table[i] = make_float2((float)c, (float)s);
}

template <typename T>
struct Row8;

template <>
struct Row8<uint16_t> {  // 8 bf16 = 16 bytes
  static __device__ __forceinline__ void load(const uint16_t* p, float* x) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));  // streamed once
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[2 * j] = bf16lo(v[j]);
      x[2 * j + 1] = bf16hi(v[j]);
    }
  }
  static __device__ __forceinline__ void store(uint16_t* p, const float* x) {
    u32x4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = pack_bf16(x[2 * j], x[2 * j + 1]);
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
  }
};

template <>
struct Row8<float> {
  static __device__ __forceinline__ void load(const float* p, float* x) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* x) {
    *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
  }
};

// X, Xout: [heads][n][d].  Thread (m, c) owns pairs 8c .. 8c+7 of position m:
//   split halves: elements 8c..8c+7 (first of each pair) and d/2 + 8c .. +7 (second),
//   adjacent pairs: elements 16c .. 16c+15, pair 8c+j = (16c+2j, 16c+2j+1).
template <typename T, bool INTERLEAVED>
__global__ __launch_bounds__(ROPE_THREADS) void rope_apply_kernel(const T* __restrict__ X, T* __restrict__ Xout,
                                                                   const float2* __restrict__ table, int heads, int n,
                                                                   int d, int inverse) {
  const int cpr = d / 16;  // threads per row
  const long t = (long)blockIdx.x * ROPE_THREADS + threadIdx.x;
  if (t >= (long)n * cpr) return;
  const int m = (int)(t / cpr), c = (int)(t % cpr);
  float cs[8], sn[8];
  {
    const float4* tp = reinterpret_cast<const float4*>(table + (size_t)m * (d / 2) + 8 * c);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 v = tp[j];
      cs[2 * j] = v.x; sn[2 * j] = v.y;
      cs[2 * j + 1] = v.z; sn[2 * j + 1] = v.w;
    }
    if (inverse) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sn[j] = -sn[j];
    }
  }
  const int h0 = blockIdx.y * ROPE_HEADS_PER_BLOCK;
  const int h1 = min(h0 + ROPE_HEADS_PER_BLOCK, heads);
  const int off_a = INTERLEAVED ? 16 * c : 8 * c;
  const int off_b = INTERLEAVED ? 16 * c + 8 : d / 2 + 8 * c;
  for (int h = h0; h < h1; ++h) {
    const size_t row = ((size_t)h * n + m) * d;
    float u[8], v[8], ou[8], ov[8];
    Row8<T>::load(X + row + off_a, u);
    Row8<T>::load(X + row + off_b, v);
    if (INTERLEAVED) {
      // u = elements 16c..16c+7 = pairs 8c..8c+3, v = pairs 8c+4..8c+7
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ou[2 * j] = u[2 * j] * cs[j] - u[2 * j + 1] * sn[j];
        ou[2 * j + 1] = u[2 * j] * sn[j] + u[2 * j + 1] * cs[j];
        ov[2 * j] = v[2 * j] * cs[4 + j] - v[2 * j + 1] * sn[4 + j];
        ov[2 * j + 1] = v[2 * j] * sn[4 + j] + v[2 * j + 1] * cs[4 + j];
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        ou[j] = u[j] * cs[j] - v[j] * sn[j];
        ov[j] = u[j] * sn[j] + v[j] * cs[j];
      }
    }
    Row8<T>::store(Xout + row + off_a, ou);
    Row8<T>::store(Xout + row + off_b, ov);
  }
}

template <typename T>
hipError_t launch_apply(const void* X, void* Xout, const float* table, int heads, int n, int d, int interleaved,
                        int inverse, hipStream_t st) {
  const long threads = (long)n * (d / 16);
  dim3 grid((unsigned)((threads + ROPE_THREADS - 1) / ROPE_THREADS),
            (unsigned)((heads + ROPE_HEADS_PER_BLOCK - 1) / ROPE_HEADS_PER_BLOCK));
  const float2* tb = reinterpret_cast<const float2*>(table);
  if (interleaved)
    rope_apply_kernel<T, true><<<grid, ROPE_THREADS, 0, st>>>((const T*)X, (T*)Xout, tb, heads, n, d, inverse);
  else
    rope_apply_kernel<T, false><<<grid, ROPE_THREADS, 0, st>>>((const T*)X, (T*)Xout, tb, heads, n, d, inverse);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_rope_table(float* table, int n, int d, double base, int pos0, hipStream_t st) {
  const long total = (long)n * (d / 2);
  rope_table_kernel<<<(unsigned)((total + ROPE_THREADS - 1) / ROPE_THREADS), ROPE_THREADS, 0, st>>>(
      reinterpret_cast<float2*>(table), n, d / 2, base, pos0);
  return hipGetLastError();
}

hipError_t launch_rope_apply(const void* X, void* Xout, const float* table, int heads, int n, int d, int bf16,
                             int interleaved, int inverse, hipStream_t st) {
  if (heads > 65535 * ROPE_HEADS_PER_BLOCK) return hipErrorNotSupported;
  return bf16 ? launch_apply<uint16_t>(X, Xout, table, heads, n, d, interleaved, inverse, st)
              : launch_apply<float>(X, Xout, table, heads, n, d, interleaved, inverse, st);
}

}  // namespace sa
