// Decoding step of the inference setting (Sec. 4.2): the sparse modes are used while the prompt is
// processed; each generated token then attends to the whole K/V cache.  One query row per (b, hq), plain
// softmax attention (Eq. 1 with every cached row visible) over rows 0..len-1.
//
// The step reads every cached K and V row once and does 4*d flop per row and query head: it is bound by
// HBM.  The cache of one KV head is cut into chunks of rows; a workgroup takes one chunk for all query
// heads of the group (so K/V rows are read once per group), keeps a running (max, sum, weighted V sum) per
// head and leaves one partial result per chunk; a second small kernel merges the partial results.
// A row of d elements is spread over d/8 lanes (16 bytes per lane for bf16), so one wave-wide load
// instruction fetches 64/(d/8) whole rows, contiguous in memory; the d/8 partial dot products are added with
// DPP moves inside a row of 16 lanes.
#include <math.h>

#include "sa_common.h"
#include "sa_device.h"

#ifndef DECODE_CHUNK
#define DECODE_CHUNK 512         // cached rows per workgroup (per-workgroup set-up and merge cost favours long chunks)
#endif
#ifndef DECODE_TARGET_WGS
#define DECODE_TARGET_WGS 512    // ... shortened (down to 64 rows) until the launch has at least this many workgroups
#endif
#ifndef DECODE_TRANSPOSED
#define DECODE_TRANSPOSED 1
#endif
#ifndef DECODE_TRANSPOSED_MIN_G
#define DECODE_TRANSPOSED_MIN_G 4
#endif
#ifndef DECODE_WAVES_PER_SIMD
#define DECODE_WAVES_PER_SIMD(T, D, G) ((sizeof(T) == 2 && (D) == 128 && (G) >= 8) ? 3 : 1)   // register budget asked of the compiler (512 / waves)
#endif
#ifndef DECODE_UNROLL
#define DECODE_UNROLL 4          // wave-wide K (and V) loads in flight per loop iteration
#endif

namespace sa {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the LPR (8 or 16) consecutive lanes that hold one row; every lane of the group gets the sum.
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror: lane i <-> 7 - i of each 8
  if (LPR == 16) v += dpp_move<0x140>(v);  // row_mirror: lane i <-> 15 - i
  return v;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

// Halving steps of a transposed sum over a row of 16 lanes (4 banks of 4).  The result is x + x(partner) in
// the lanes of one half of the banks and y + y(partner) in the other half: each lane gives one of its two values
// away and keeps the other, so two values cost two instructions instead of four.  A DPP instruction must not
// read a register in the two issue slots after a vector instruction wrote it, and the compiler does not look
// inside the block: hence the waits at both ends.
__device__ __forceinline__ float add_split_mirror(float x, float y) {        // partner 15 - i; banks {0,1} | {2,3}
  float r;
  asm("s_nop 1\n\t"
      "v_add_f32_dpp %0, %1, %1 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %0, %2, %2 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "s_nop 1"
      : "=&v"(r) : "v"(x), "v"(y));
  return r;
}
__device__ __forceinline__ float add_split_half_mirror(float x, float y) {   // partner 7 - i of each 8; banks {0,2} | {1,3}
  float r;
  asm("s_nop 1\n\t"
      "v_add_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
      "v_add_f32_dpp %0, %2, %2 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
      "s_nop 1"
      : "=&v"(r) : "v"(x), "v"(y));
  return r;
}

__device__ __forceinline__ void load8(const bf16_t* p, float (&out)[8]) {
  const u32x4 r = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = bf16lo(r[i]);
    out[2 * i + 1] = bf16hi(r[i]);
  }
}

__device__ __forceinline__ void load8(const float* p, float (&out)[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[i] = a[i];
    out[4 + i] = b[i];
  }
}

__device__ __forceinline__ void store1(bf16_t* p, float v) {
  *reinterpret_cast<uint16_t*>(p) = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
}
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }

struct Args {
  const void* q;
  const void* K;
  const void* V;
  float* part;      // [B*Hq][splits][d + 2]: weighted V sum, then running max (log2 domain) and sum
  const int32_t* lens;   // per-sequence row counts [B] or nullptr (then every sequence has `len` rows)
  int Hq, Hkv, g, n, len, chunk, splits;
  float scale_log2e;
};

// exp2(a - b) where b is the reference maximum; a = b = -inf (nothing seen yet) gives 0
__device__ __forceinline__ float exp2_rel(float a, float ref) { return exp2f(a - (ref == -INFINITY ? 0.f : ref)); }

// Per-lane state of one lane group: the slice of 8 elements of the query rows, the running maximum (log2
// domain), the running sum and the weighted V sum of every head.  The bf16 form keeps rows as packed pairs and
// uses the two-element dot product instruction for both products (the weights are rounded to bf16 for the
// second one, as in the prefill kernels); the fp32 form uses plain multiply-adds.
template <typename T, int G, int U>
struct Lane;

template <int G, int U>
struct Lane<float, G, U> {
  float qf[G][8];
  float kx[U][8], vx[U][8];
  __device__ __forceinline__ void load_q(const float* p, int h, float scale_log2e) {
    load8(p, qf[h]);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[h][e] *= scale_log2e;
  }
  __device__ __forceinline__ void load_row(const float* k, const float* v, int u) {
    load8(k, kx[u]);
    load8(v, vx[u]);
  }
  __device__ __forceinline__ float partial_score(int h, int u) const {
    float dot = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) dot = fmaf(qf[h][e], kx[u][e], dot);
    return dot;
  }
  static __device__ __forceinline__ float finish_score(float dot, float) { return dot; }
  // acc = acc * corr + sum_u p[u] * V_u; returns sum_u p[u]
  __device__ __forceinline__ float accumulate(float (&acc)[8], float corr, const float (&p)[U]) const {
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) psum += p[u];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[e] * corr;
#pragma unroll
      for (int u = 0; u < U; ++u) v = fmaf(p[u], vx[u][e], v);
      acc[e] = v;
    }
    return psum;
  }
};

template <int G, int U>
struct Lane<bf16_t, G, U> {
  static_assert(U % 2 == 0, "rows are consumed in pairs");
  u32x4 q2[G];
  u32x4 kx[U], vx[U];
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
  }
  __device__ __forceinline__ void load_q(const bf16_t* p, int h, float) { q2[h] = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ void load_row(const bf16_t* k, const bf16_t* v, int u) {
    kx[u] = *reinterpret_cast<const u32x4*>(k);
    vx[u] = *reinterpret_cast<const u32x4*>(v);
  }
  __device__ __forceinline__ float partial_score(int h, int u) const {
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) dot = dot2(q2[h][i], kx[u][i], dot);
    return dot;
  }
  static __device__ __forceinline__ float finish_score(float dot, float scale_log2e) { return dot * scale_log2e; }
  // acc = acc * corr + sum_u w[u] * V_u with the weights as bf16 pairs pp[u/2] = (w[u], w[u+1])
  __device__ __forceinline__ void accumulate_packed(float (&acc)[8], float corr, const uint32_t (&pp)[U / 2]) const {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= corr;
#pragma unroll
    for (int u = 0; u < U; u += 2) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // (V_u[2i], V_u+1[2i]) and (V_u[2i+1], V_u+1[2i+1])
        const uint32_t even = __builtin_amdgcn_perm(vx[u + 1][i], vx[u][i], 0x05040100u);
        const uint32_t odd = __builtin_amdgcn_perm(vx[u + 1][i], vx[u][i], 0x07060302u);
        acc[2 * i] = dot2(even, pp[u / 2], acc[2 * i]);
        acc[2 * i + 1] = dot2(odd, pp[u / 2], acc[2 * i + 1]);
      }
    }
  }
  __device__ __forceinline__ float accumulate(float (&acc)[8], float corr, const float (&p)[U]) const {
    float psum = 0.f;
    uint32_t pp[U / 2];
#pragma unroll
    for (int u = 0; u < U; u += 2) {
      pp[u / 2] = pack_bf16(p[u], p[u + 1]);
      psum += bf16lo(pp[u / 2]) + bf16hi(pp[u / 2]);
    }
    accumulate_packed(acc, corr, pp);
    return psum;
  }
};

template <typename T, int D, int G>
__global__ __launch_bounds__(kThreads, DECODE_WAVES_PER_SIMD(T, D, G)) void decode_partial_kernel(Args a) {
  constexpr int LPR = D / 8;          // lanes per row
  constexpr int KPW = 64 / LPR;       // rows per wave-wide load
  constexpr int STEP = kWaves * KPW;  // rows per workgroup per load
  constexpr int U = DECODE_UNROLL;
  // bf16 rows over 16 lanes, four loads per iteration: one load per bank of a DPP row
  constexpr bool kTransposed = DECODE_TRANSPOSED && sizeof(T) == 2 && LPR == 16 && U == 4 && G >= DECODE_TRANSPOSED_MIN_G;
  __shared__ float lds_acc[kWaves][G][D];
  __shared__ float lds_ml[kWaves][G][2];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPR, sub = lane % LPR;
  const int split = blockIdx.x;
  const int gsets = a.g / G;
  const int set = blockIdx.y % gsets, bhk = blockIdx.y / gsets;
  const int hk = bhk % a.Hkv, b = bhk / a.Hkv;
  const int hq0 = hk * a.g + set * G;
  const size_t head_off = ((size_t)b * a.Hkv + hk) * (size_t)a.n * D + sub * 8;
  const T* Kh = reinterpret_cast<const T*>(a.K) + head_off;
  const T* Vh = reinterpret_cast<const T*>(a.V) + head_off;

  Lane<T, G, U> st;
  float acc[G][8], m[G], l[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    st.load_q(reinterpret_cast<const T*>(a.q) + ((size_t)b * a.Hq + hq0 + h) * D + sub * 8, h, a.scale_log2e);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
    m[h] = -INFINITY;
    l[h] = 0.f;
  }

  const int k0 = split * a.chunk;
  // the launch covers `len` rows; a sequence with fewer rows (clamped to 1..len) leaves its last chunks empty
  const int len_b = a.lens ? min(max(a.lens[b], 1), a.len) : a.len;
  const int k1 = min(len_b, k0 + a.chunk);
  if (k0 >= k1) {   // uniform over the workgroup: an empty chunk contributes weight zero to the merge
    for (int idx = threadIdx.x; idx < G * (D + 2); idx += kThreads) {
      const int h = idx / (D + 2), e = idx % (D + 2);
      a.part[(((size_t)b * a.Hq + hq0 + h) * a.splits + split) * (D + 2) + e] = e == D ? -INFINITY : 0.f;
    }
    return;
  }
  for (int it = k0; it < k1; it += STEP * U) {
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = it + u * STEP + wave * KPW + grp;
      valid[u] = j < k1;
      const size_t row = (size_t)(valid[u] ? j : k1 - 1) * D;   // rows past the chunk re-read its last row
      st.load_row(Kh + row, Vh + row, u);
    }
    if constexpr (kTransposed) {
      // Bank b of a row of 16 lanes ends up with the scores of load u = b only (all G heads), computes their
      // weights once instead of in all 16 lanes, and the four banks exchange the weights as bf16 pairs.
      const int bank = (lane >> 2) & 3;
      const bool own_valid = it + bank * STEP + wave * KPW + grp < k1;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float r0 = add_split_mirror(st.partial_score(h, 0), st.partial_score(h, 2));   // banks 0,1: u = 0 | banks 2,3: u = 2
        const float r1 = add_split_mirror(st.partial_score(h, 1), st.partial_score(h, 3));   //            u = 1 |            u = 3
        float t = add_split_half_mirror(r0, r1);                                             // bank b: u = b
        t += dpp_move<0xB1>(t);
        t += dpp_move<0x4E>(t);
        const float own = own_valid ? t * a.scale_log2e : -INFINITY;
        float mn = fmaxf(own, dpp_move<0x140>(own));
        mn = fmaxf(mn, dpp_move<0x141>(mn));
        mn = fmaxf(mn, m[h]);
        const float corr = exp2_rel(m[h], mn);
        const float w = exp2_rel(own, mn);
        m[h] = mn;
        // (own, neighbour bank's) -> (even bank's, odd bank's); then the other pair from the mirrored bank
        uint32_t pair = pack_bf16(w, dpp_move<0x141>(w));
        l[h] = fmaf(l[h], corr, bf16lo(pair));             // this bank's share; the banks are summed after the loop
        pair = __builtin_amdgcn_alignbit(pair, pair, (bank & 1) ? 16u : 0u);
        const uint32_t other = dpp_move_u32<0x140>(pair);
        const uint32_t pp[2] = {bank < 2 ? pair : other, bank < 2 ? other : pair};
        st.accumulate_packed(acc[h], corr, pp);
      }
      continue;
    }
    float s[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float dot = st.finish_score(row_sum<LPR>(st.partial_score(h, u)), a.scale_log2e);
        s[u][h] = valid[u] ? dot : -INFINITY;
      }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mn = m[h];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][h]);
      const float corr = exp2_rel(m[h], mn);
      float p[U];
#pragma unroll
      for (int u = 0; u < U; ++u) p[u] = exp2_rel(s[u][h], mn);
      const float psum = st.accumulate(acc[h], corr, p);
      l[h] = fmaf(l[h], corr, psum);
      m[h] = mn;
    }
  }

  if constexpr (kTransposed) {   // every bank of a row kept its own share of the sums
#pragma unroll
    for (int h = 0; h < G; ++h) {
      l[h] += dpp_move<0x140>(l[h]);
      l[h] += dpp_move<0x141>(l[h]);
    }
  }
  // merge the KPW lane groups of the wave (same `sub`, different rows)
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mw = m[h];
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
    const float c = exp2_rel(m[h], mw);
    float lw = l[h] * c;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) lw += __shfl_xor(lw, off);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[h][e] * c;
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) v += __shfl_xor(v, off);
      acc[h][e] = v;
    }
    if (grp == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) lds_acc[wave][h][sub * 8 + e] = acc[h][e];
      if (sub == 0) {
        lds_ml[wave][h][0] = mw;
        lds_ml[wave][h][1] = lw;
      }
    }
  }
  __syncthreads();

  // merge the waves; at least one of them saw a row, so the maximum is finite
  for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
    const int h = idx / D, e = idx % D;
    float M = lds_ml[0][h][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, lds_ml[w][h][0]);
    float v = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float c = exp2f(lds_ml[w][h][0] - M);
      v = fmaf(c, lds_acc[w][h][e], v);
      L = fmaf(c, lds_ml[w][h][1], L);
    }
    float* out = a.part + (((size_t)b * a.Hq + hq0 + h) * a.splits + split) * (D + 2);
    out[e] = v;
    if (e == 0) {
      out[D] = M;
      out[D + 1] = L;
    }
  }
}

// One workgroup per (b, hq): merges the partial results of the chunks.  The rows of the partial results are
// spread over 16 waves, so that even a cache cut into hundreds of chunks costs a few dependent steps.
constexpr int kMergeWaves = 16;

template <typename T, int D>
__global__ __launch_bounds__(kMergeWaves * 64) void decode_merge_kernel(const float* __restrict__ part,
                                                                        T* __restrict__ Y, float* __restrict__ LSE,
                                                                        int splits) {
  constexpr int EPL = (D + 63) / 64;   // elements per lane
  __shared__ float lds_m[kMergeWaves];
  __shared__ float lds_acc[kMergeWaves][D + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* P = part + (size_t)blockIdx.x * splits * (D + 2);

  float M = -INFINITY;
  for (int s = threadIdx.x; s < splits; s += kMergeWaves * 64) M = fmaxf(M, P[(size_t)s * (D + 2) + D]);
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
  if (lane == 0) lds_m[wave] = M;
  __syncthreads();
  M = lds_m[0];
#pragma unroll
  for (int w = 1; w < kMergeWaves; ++w) M = fmaxf(M, lds_m[w]);

  float acc[EPL] = {}, L = 0.f;
#pragma unroll 4   // independent rows: keep several loads in flight
  for (int s = wave; s < splits; s += kMergeWaves) {
    const float* row = P + (size_t)s * (D + 2);
    const float c = exp2f(row[D] - M);
    L = fmaf(c, row[D + 1], L);
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = fmaf(c, row[lane + 64 * i], acc[i]);
  }
#pragma unroll
  for (int i = 0; i < EPL; ++i) lds_acc[wave][lane + 64 * i] = acc[i];
  if (lane == 0) lds_acc[wave][D] = L;
  __syncthreads();
  if (threadIdx.x < D) {
    const int e = threadIdx.x;
    float Lt = 0.f, v = 0.f;
#pragma unroll
    for (int w = 0; w < kMergeWaves; ++w) {
      Lt += lds_acc[w][D];
      v += lds_acc[w][e];
    }
    store1(Y + (size_t)blockIdx.x * D + e, v / Lt);
    if (e == 0 && LSE) LSE[blockIdx.x] = (M + log2f(Lt)) * kLn2;
  }
}

int heads_per_workgroup(int g) { return g % 8 == 0 ? 8 : (g % 4 == 0 ? 4 : (g % 2 == 0 ? 2 : 1)); }

// Rows per chunk, fixed by the capacity n so that the workspace bound holds for every len <= n.
int chunk_rows(int B, int Hkv, int g, int n) {
  const long long groups = (long long)B * Hkv * (g / heads_per_workgroup(g));
  int chunk = DECODE_CHUNK;
  while (chunk > 64 && ((long long)(n + chunk - 1) / chunk) * groups < DECODE_TARGET_WGS) chunk >>= 1;
  return chunk;
}

template <typename T, int D, int G>
hipError_t launch_typed(const Decode& d, const Args& a, hipStream_t st) {
  const int gsets = a.g / G;
  dim3 grid((unsigned)a.splits, (unsigned)(d.B * d.Hkv * gsets));
  decode_partial_kernel<T, D, G><<<grid, kThreads, 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  decode_merge_kernel<T, D><<<d.B * d.Hq, kMergeWaves * 64, 0, st>>>(a.part, reinterpret_cast<T*>(d.Y), d.LSE, a.splits);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_heads(const Decode& d, const Args& a, hipStream_t st) {
  switch (heads_per_workgroup(a.g)) {
    case 8: return launch_typed<T, D, 8>(d, a, st);
    case 4: return launch_typed<T, D, 4>(d, a, st);
    case 2: return launch_typed<T, D, 2>(d, a, st);
    default: return launch_typed<T, D, 1>(d, a, st);
  }
}

}  // namespace

size_t decode_workspace_bytes(int B, int Hq, int Hkv, int n, int d) {
  const int chunk = chunk_rows(B, Hkv, Hq / Hkv, n);
  const size_t splits = (size_t)(n + chunk - 1) / chunk;
  return (size_t)B * Hq * splits * (d + 2) * sizeof(float);
}

hipError_t launch_decode(const Decode& d, hipStream_t st) {
  if (!(d.d == 64 || d.d == 128) || d.len < 1 || d.len > d.n || d.Hq % d.Hkv != 0) return hipErrorInvalidValue;
  Args a;
  a.q = d.q; a.K = d.K; a.V = d.V;
  a.part = d.part;
  a.lens = d.lens;
  a.Hq = d.Hq; a.Hkv = d.Hkv; a.g = d.Hq / d.Hkv; a.n = d.n; a.len = d.len;
  a.chunk = chunk_rows(d.B, d.Hkv, a.g, d.n);
  a.splits = (d.len + a.chunk - 1) / a.chunk;
  a.scale_log2e = d.scale * kLog2e;
  if ((long long)d.B * d.Hkv * a.g > 65535) return hipErrorInvalidValue;   // grid.y
  if (d.bf16) return d.d == 64 ? launch_heads<bf16_t, 64>(d, a, st) : launch_heads<bf16_t, 128>(d, a, st);
  return d.d == 64 ? launch_heads<float, 64>(d, a, st) : launch_heads<float, 128>(d, a, st);
}

}  // namespace sa
