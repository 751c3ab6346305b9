// Element-wise helpers of libsa: permutation check, zero fill, and the backward's preparation pass
// (D = rowsum(dO * O), and for the gated sum of Eq. 5 the chain rule through the two sigmoid gates).
#include "sa_common.h"
#include "sa_device.h"

namespace sa {
namespace {

__global__ void fill_zero_kernel(uint32_t* p, size_t words) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < words; i += stride) p[i] = 0u;
}

// seen[slice][v] counts how often value v occurs in the slice; any count other than one, or a value
// outside 0..n-1, raises the flag.
__global__ void check_perm_kernel(const int32_t* __restrict__ perm, size_t total, int n, int* seen, int* flag) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < total; i += stride) {
    const int v = perm[i];
    if (v < 0 || v >= n) {
      atomicOr(flag, 1);
    } else if (atomicAdd(&seen[(i / n) * n + v], 1) != 0) {
      atomicOr(flag, 1);
    }
  }
}

// The gather and the scatter of Alg. 1 without the attention in between (a measurement helper: the
// ceiling for rows of 2*d bytes addressed through the index tensor).  One group of LPR lanes per
// (b, hq, slot): Y[perm[p]] = Q[perm[p]] (+ K[perm[p]] + V[perm[p]] for the first query head of a KV
// group, so that every K and V row is read once per group as in the attention kernels).  Four rows
// per thread are in flight.
template <int LPR>
__global__ __launch_bounds__(256) void permuted_copy_bf16_kernel(const Pass p, const long rows) {
  constexpr int RPT = 4;
  const int sub = threadIdx.x % LPR;
  const long group = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
  const long groups = (long)gridDim.x * 256 / LPR;
  const int d = LPR * 8;
  for (long r0 = group; r0 < rows; r0 += groups * RPT) {
    long r[RPT];
    int src[RPT];
    bool ok[RPT];
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
      r[j] = r0 + j * groups;
      ok[j] = r[j] < rows;
      const long rr = ok[j] ? r[j] : 0;
      const int slot = (int)(rr % p.n);
      const long bh = rr / p.n;
      const int hq = (int)(bh % p.Hq), b = (int)(bh / p.Hq);
      src[j] = p.perm ? p.perm[(size_t)perm_slice_index(p.perm_B, p.perm_H, b, hq) * p.n + slot] : slot;
    }
    u32x4 q[RPT], k[RPT], v[RPT];
    bool lead[RPT];
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
      const long rr = ok[j] ? r[j] : 0;
      const long bh = rr / p.n;
      const int hq = (int)(bh % p.Hq), b = (int)(bh / p.Hq);
      lead[j] = hq % p.g == 0;
      const size_t qoff = ((size_t)bh * p.n + src[j]) * d + sub * 8;
      const size_t koff = (((size_t)b * p.Hkv + hq / p.g) * p.n + src[j]) * d + sub * 8;
      // every row is touched once: non-temporal loads and stores
      q[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.Q) + qoff));
      if (lead[j]) {
        k[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.K) + koff));
        v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.V) + koff));
      }
    }
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
      if (!ok[j]) continue;
      u32x4 o = q[j];
      if (lead[j]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          o[e] = pack_bf16(bf16lo(q[j][e]) + bf16lo(k[j][e]) + bf16lo(v[j][e]),
                           bf16hi(q[j][e]) + bf16hi(k[j][e]) + bf16hi(v[j][e]));
      }
      const size_t qoff = ((size_t)(r[j] / p.n) * p.n + src[j]) * d + sub * 8;
      __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.Y) + qoff));
    }
  }
}

// ---- permutation sampler (Sec. 3.3: sigma ~ Uniform(S_n), fresh per layer): sort by random key.
// Slot p of slice s gets the 64-bit sort key  (r(p) with its low 20 bits replaced by p),  r(p) = the
// (p+1)-th output of SplitMix64 started at a per-(seed, layer, slice) stream value: 44 random bits,
// ties broken by p, all keys distinct.  perm = argsort of the keys, computed as a rank: the thread of
// slot p counts the keys below its own and writes perm[rank] = p.  All keys of the slice stream
// through LDS in tiles of 1024; 16 lanes share one slot (each takes every 16th pair of keys of a
// tile, the partial counts are added with shuffles), so even a short slice fills the chip.
__device__ __forceinline__ uint64_t splitmix_mix(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kIndexMask = 0xFFFFFull;  // n <= 2^20
constexpr int SAMPLE_TILE = 1024;

__device__ __forceinline__ uint64_t sort_key(uint64_t stream, int p) {
  return (splitmix_mix(stream + kGamma * (uint64_t)(p + 1)) & ~kIndexMask) | (uint64_t)p;
}

constexpr int SAMPLE_LPP = 16;  // lanes that share the rank count of one slot

__global__ __launch_bounds__(256) void sample_perm_kernel(int32_t* __restrict__ perm, const int n, const uint64_t seed,
                                                           const int layer) {
  __shared__ __attribute__((aligned(16))) uint64_t tile[SAMPLE_TILE];
  const int slice = blockIdx.y;
  const uint64_t stream = splitmix_mix(splitmix_mix(seed) + kGamma * (((uint64_t)(uint32_t)layer << 32) | (uint32_t)slice));
  const int p = blockIdx.x * (256 / SAMPLE_LPP) + threadIdx.x / SAMPLE_LPP;
  const int sub = threadIdx.x % SAMPLE_LPP;
  const uint64_t mine = sort_key(stream, p);
  int rank = 0;
  for (int q0 = 0; q0 < n; q0 += SAMPLE_TILE) {
    __syncthreads();
    // keys past the end of the slice are set above every real key
    for (int j = threadIdx.x; j < SAMPLE_TILE; j += 256) tile[j] = q0 + j < n ? sort_key(stream, q0 + j) : ~0ull;
    __syncthreads();
#pragma unroll 8
    for (int j = 2 * sub; j < SAMPLE_TILE; j += 2 * SAMPLE_LPP) {  // two keys per 16-byte read
      const ulonglong2 k = *reinterpret_cast<const ulonglong2*>(tile + j);
      rank += (k.x < mine) ? 1 : 0;
      rank += (k.y < mine) ? 1 : 0;
    }
  }
#pragma unroll
  for (int o = SAMPLE_LPP / 2; o > 0; o >>= 1) rank += __shfl_xor(rank, o);
  if (sub == 0 && p < n) perm[(size_t)slice * n + rank] = p;
}

// ---- the same permutation in O(n) work, with a workspace: the keys are uniform 64-bit numbers, so their
// top bits spread them evenly over NB buckets (64 keys each on average).  Count per bucket, exclusive scan,
// scatter the keys into their buckets (in any order), then rank every key inside its bucket: the slot of
// key k goes to perm[start(bucket) + #{keys of the bucket below k}].  The result does not depend on the
// order in which the atomic counters hand out places.
__device__ __forceinline__ uint64_t slice_stream(uint64_t seed, int layer, int slice) {
  return splitmix_mix(splitmix_mix(seed) + kGamma * (((uint64_t)(uint32_t)layer << 32) | (uint32_t)slice));
}

struct SampleWs {
  uint64_t* keys;  // [slices][n]
  int* count;      // [slices][NB]
  int* cursor;     // [slices][NB]: first free place of the bucket while scattering, its end afterwards
  int NB, shift;   // bucket of key k = k >> shift (shift = 64: one bucket)
};

__device__ __forceinline__ int bucket_of(uint64_t k, int shift) { return shift >= 64 ? 0 : (int)(k >> shift); }

__global__ __launch_bounds__(256) void sample_count_kernel(SampleWs w, const int n, const uint64_t seed, const int layer) {
  const int slice = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= n) return;
  const uint64_t k = sort_key(slice_stream(seed, layer, slice), p);
  atomicAdd(w.count + (size_t)slice * w.NB + bucket_of(k, w.shift), 1);
}

// one workgroup per slice: cursor = exclusive prefix sum of count
__global__ __launch_bounds__(256) void sample_scan_kernel(SampleWs w) {
  __shared__ int part[256];
  const int slice = blockIdx.x, t = threadIdx.x;
  const int* cnt = w.count + (size_t)slice * w.NB;
  int* cur = w.cursor + (size_t)slice * w.NB;
  const int per = (w.NB + 255) / 256, b0 = t * per, b1 = min(b0 + per, w.NB);
  int sum = 0;
  for (int b = b0; b < b1; ++b) sum += cnt[b];
  part[t] = sum;
  __syncthreads();
  if (t == 0) {
    int run = 0;
    for (int i = 0; i < 256; ++i) {
      const int v = part[i];
      part[i] = run;
      run += v;
    }
  }
  __syncthreads();
  int run = part[t];
  for (int b = b0; b < b1; ++b) {
    cur[b] = run;
    run += cnt[b];
  }
}

__global__ __launch_bounds__(256) void sample_scatter_kernel(SampleWs w, const int n, const uint64_t seed, const int layer) {
  const int slice = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= n) return;
  const uint64_t k = sort_key(slice_stream(seed, layer, slice), p);
  const int place = atomicAdd(w.cursor + (size_t)slice * w.NB + bucket_of(k, w.shift), 1);
  w.keys[(size_t)slice * n + place] = k;
}

__global__ __launch_bounds__(256) void sample_rank_kernel(SampleWs w, int32_t* __restrict__ perm, const int n) {
  const int slice = blockIdx.y, e = blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  const uint64_t* keys = w.keys + (size_t)slice * n;
  const uint64_t k = keys[e];
  const int b = bucket_of(k, w.shift);
  const int cnt = w.count[(size_t)slice * w.NB + b];
  const int start = w.cursor[(size_t)slice * w.NB + b] - cnt;  // the cursor ended at the bucket's end
  int rank = 0;
  for (int j = 0; j < cnt; ++j) rank += keys[start + j] < k ? 1 : 0;
  perm[(size_t)slice * n + start + rank] = (int32_t)(k & kIndexMask);
}

template <int LPR>  // lanes per row, each lane owns 16 bytes of the row
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One group of LPR lanes per row; E = elements per 16-byte vector (8 bf16 / 4 f32).
template <bool BF16, int LPR>
__global__ __launch_bounds__(256) void bwd_prepare_kernel(Prep p) {
  constexpr int E = BF16 ? 8 : 4;
  const int sub = threadIdx.x % LPR;
  const long row = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
  const bool valid = row < p.rows;
  const size_t r = valid ? (size_t)row : 0;
  const size_t off = r * p.d + (size_t)sub * E;

  float dy[E], ya[E], yb[E];
  if (BF16) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.dY) + off);
    const u32x4 b = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.Y_a) + off);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      dy[2 * k] = bf16lo(a[k]); dy[2 * k + 1] = bf16hi(a[k]);
      ya[2 * k] = bf16lo(b[k]); ya[2 * k + 1] = bf16hi(b[k]);
    }
    if (p.gated) {
      const u32x4 c = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.Y_b) + off);
#pragma unroll
      for (int k = 0; k < 4; ++k) { yb[2 * k] = bf16lo(c[k]); yb[2 * k + 1] = bf16hi(c[k]); }
    }
  } else {
    const f32x4 a = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.dY) + off);
    const f32x4 b = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.Y_a) + off);
#pragma unroll
    for (int k = 0; k < 4; ++k) { dy[k] = a[k]; ya[k] = b[k]; }
    if (p.gated) {
      const f32x4 c = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.Y_b) + off);
#pragma unroll
      for (int k = 0; k < 4; ++k) yb[k] = c[k];
    }
  }

  if (!p.gated) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < E; ++k) s = fmaf(dy[k], ya[k], s);
    s = group_sum<LPR>(s);
    if (valid && sub == 0) p.D_a[r] = s;
    return;
  }

  // gated: dO_x = sig(gamma_x) * dY;  D_x = sum_d dO_x * Y_x;  dgamma_x = sig'(gamma_x) * dY * Y_x
  float ga[E], gb[E];
  if (p.gate_per_dim) {
#pragma unroll
    for (int k = 0; k < E; ++k) {
      ga[k] = sigmoidf_exact(load_gate(p.gate_a, off + k, p.gate_f32));
      gb[k] = sigmoidf_exact(load_gate(p.gate_b, off + k, p.gate_f32));
    }
  } else {  // one gate per row: one sigmoid, not one per element
    const float a1 = sigmoidf_exact(load_gate(p.gate_a, r, p.gate_f32));
    const float b1 = sigmoidf_exact(load_gate(p.gate_b, r, p.gate_f32));
#pragma unroll
    for (int k = 0; k < E; ++k) {
      ga[k] = a1;
      gb[k] = b1;
    }
  }
  float da[E], db[E], sa = 0.f, sb = 0.f, ra = 0.f, rb = 0.f;
#pragma unroll
  for (int k = 0; k < E; ++k) {
    da[k] = ga[k] * dy[k];
    db[k] = gb[k] * dy[k];
    sa = fmaf(da[k], ya[k], sa);
    sb = fmaf(db[k], yb[k], sb);
    ra = fmaf(dy[k], ya[k], ra);
    rb = fmaf(dy[k], yb[k], rb);
  }
  if (p.fold) {  // one gate per row: E_x, LSE_x - ln g_x, dgamma_x; no copy of dY
    ra = group_sum<LPR>(ra);
    rb = group_sum<LPR>(rb);
    if (valid && sub == 0) {
      const float xa = load_gate(p.gate_a, r, p.gate_f32), xb = load_gate(p.gate_b, r, p.gate_f32);
      // -ln sigmoid(x) = ln(1 + e^-x), evaluated without cancellation on either side
      const float na = xa > 0.f ? log1pf(__expf(-xa)) : -xa + log1pf(__expf(xa));
      const float nb = xb > 0.f ? log1pf(__expf(-xb)) : -xb + log1pf(__expf(xb));
      p.D_a[r] = ra;
      p.D_b[r] = rb;
      p.L_a[r] = p.lse_a[r] + na;
      p.L_b[r] = p.lse_b[r] + nb;
      store_gate(p.dgate_a, r, p.gate_f32, ga[0] * (1.f - ga[0]) * ra);
      store_gate(p.dgate_b, r, p.gate_f32, gb[0] * (1.f - gb[0]) * rb);
    }
    return;
  }
  sa = group_sum<LPR>(sa);
  sb = group_sum<LPR>(sb);
  if (valid && sub == 0) {
    p.D_a[r] = sa;
    p.D_b[r] = sb;
  }
  if (p.gate_per_dim) {
    if (valid) {
#pragma unroll
      for (int k = 0; k < E; ++k) {
        store_gate(p.dgate_a, off + k, p.gate_f32, ga[k] * (1.f - ga[k]) * dy[k] * ya[k]);
        store_gate(p.dgate_b, off + k, p.gate_f32, gb[k] * (1.f - gb[k]) * dy[k] * yb[k]);
      }
    }
  } else {
    ra = group_sum<LPR>(ra);
    rb = group_sum<LPR>(rb);
    if (valid && sub == 0) {
      store_gate(p.dgate_a, r, p.gate_f32, ga[0] * (1.f - ga[0]) * ra);
      store_gate(p.dgate_b, r, p.gate_f32, gb[0] * (1.f - gb[0]) * rb);
    }
  }
  if (valid) {
    if (BF16) {
      u32x4 oa, ob;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        oa[k] = pack_bf16(da[2 * k], da[2 * k + 1]);
        ob[k] = pack_bf16(db[2 * k], db[2 * k + 1]);
      }
      *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.dO_a) + off) = oa;
      *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.dO_b) + off) = ob;
    } else {
      f32x4 oa, ob;
#pragma unroll
      for (int k = 0; k < 4; ++k) { oa[k] = da[k]; ob[k] = db[k]; }
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.dO_a) + off) = oa;
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.dO_b) + off) = ob;
    }
  }
}

template <bool BF16, int LPR>
hipError_t launch_prepare_t(const Prep& p, hipStream_t st) {
  const long threads = (long)p.rows * LPR;
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  hipLaunchKernelGGL((bwd_prepare_kernel<BF16, LPR>), dim3(blocks), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st) {
  if (bytes % 4 != 0) return hipErrorInvalidValue;
  const size_t words = bytes / 4;
  if (words == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((words + 1023) / 1024 < 4096 ? (words + 1023) / 1024 : 4096);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<uint32_t*>(ptr), words);
  return hipGetLastError();
}

hipError_t launch_check_perm(const int32_t* perm, int slices, int n, int* seen, int* flag, hipStream_t st) {
  const size_t total = (size_t)slices * n;
  hipError_t e = launch_fill_zero(seen, total * sizeof(int), st);
  if (e != hipSuccess) return e;
  e = launch_fill_zero(flag, sizeof(int), st);
  if (e != hipSuccess) return e;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
  hipLaunchKernelGGL(check_perm_kernel, dim3(blocks), dim3(256), 0, st, perm, total, n, seen, flag);
  return hipGetLastError();
}

// buckets for the workspace path: a power of two, 64 keys per bucket on average
static int sample_buckets(int n) {
  int nb = 1;
  while ((long)nb * 64 < n) nb *= 2;
  return nb;
}

size_t sample_perm_workspace_bytes(int slices, int n) {
  const size_t nb = (size_t)sample_buckets(n);
  return (size_t)slices * ((size_t)n * 8 + 2 * nb * 4) + 512;
}

hipError_t launch_sample_perm(int32_t* perm, int slices, int n, uint64_t seed, int layer, void* ws, hipStream_t st) {
  if (!perm || slices < 1 || slices > 65535 || n < 1) return hipErrorInvalidValue;
  if (n > (1 << 20)) return hipErrorNotSupported;  // the slot index takes the low 20 bits of the sort key
  // five small launches: below ~16K slots the single O(n^2) launch is faster (0.017 against 0.037 ms at
  // n = 8192; 0.135 against 0.045 ms at n = 32768)
  if (ws && n >= 16384) {
    SampleWs w;
    w.NB = sample_buckets(n);
    int bits = 0;
    while ((1 << bits) < w.NB) ++bits;
    w.shift = 64 - bits;
    char* base = reinterpret_cast<char*>((reinterpret_cast<uintptr_t>(ws) + 255) & ~(uintptr_t)255);
    w.keys = reinterpret_cast<uint64_t*>(base);
    w.count = reinterpret_cast<int*>(base + (size_t)slices * n * 8);
    w.cursor = w.count + (size_t)slices * w.NB;
    hipError_t e = launch_fill_zero(w.count, (size_t)slices * w.NB * 4, st);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((n + 255) / 256), (unsigned)slices);
    hipLaunchKernelGGL(sample_count_kernel, grid, dim3(256), 0, st, w, n, seed, layer);
    hipLaunchKernelGGL(sample_scan_kernel, dim3((unsigned)slices), dim3(256), 0, st, w);
    hipLaunchKernelGGL(sample_scatter_kernel, grid, dim3(256), 0, st, w, n, seed, layer);
    hipLaunchKernelGGL(sample_rank_kernel, grid, dim3(256), 0, st, w, perm, n);
    return hipGetLastError();
  }
  const int per_block = 256 / SAMPLE_LPP;
  hipLaunchKernelGGL(sample_perm_kernel, dim3((unsigned)((n + per_block - 1) / per_block), (unsigned)slices), dim3(256), 0, st,
                     perm, n, seed, layer);
  return hipGetLastError();
}

hipError_t launch_permuted_copy_bf16(const Pass& p, hipStream_t st) {
  if (p.n < 1 || p.B < 1 || p.Hq < 1 || p.Hkv < 1 || p.g * p.Hkv != p.Hq || !p.Q || !p.K || !p.V || !p.Y)
    return hipErrorInvalidValue;
  if (!(p.d == 64 || p.d == 128)) return hipErrorNotSupported;
  const long rows = (long)p.B * p.Hq * p.n;
  const int lpr = p.d / 8;
  const long want = (rows * lpr + 256 * 4 - 1) / (256 * 4);  // four rows per lane group
  const unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 0x7fffffffL ? 0x7fffffffL : want));
  if (p.d == 64) hipLaunchKernelGGL(permuted_copy_bf16_kernel<8>, dim3(blocks), dim3(256), 0, st, p, rows);
  else hipLaunchKernelGGL(permuted_copy_bf16_kernel<16>, dim3(blocks), dim3(256), 0, st, p, rows);
  return hipGetLastError();
}

hipError_t launch_bwd_prepare(const Prep& p, hipStream_t st) {
  if (p.rows < 1 || !(p.d == 64 || p.d == 128)) return hipErrorInvalidValue;
  if (p.bf16) return p.d == 64 ? launch_prepare_t<true, 8>(p, st) : launch_prepare_t<true, 16>(p, st);
  return p.d == 64 ? launch_prepare_t<false, 16>(p, st) : launch_prepare_t<false, 32>(p, st);
}

}  // namespace sa
