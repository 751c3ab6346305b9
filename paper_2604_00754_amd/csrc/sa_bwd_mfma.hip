// bf16 backward of Stochastic Attention on gfx950 matrix cores.
//
// The paper trains through the layer with autograd (Sec. 4.1, Table 3 times forward+backward); the
// kernels here are the analytic gradient of Eq. 1 over the visible set of Eq. 3 / App. B, in
// permuted order, with rows gathered from and scattered to their original positions:
//   P = exp(S - LSE),  dV = P^T dO,  dP = dO V^T,  dS = P * (dP - D),  dQ = scale dS K,
//   dK = scale dS^T Q,  D = rowsum(dO * O).
// Two kernels, both recomputing S from Q and K:
//   dQ kernel    -- a workgroup owns 128 query slots (as in the forward) and walks key tiles;
//                   S^T and dP^T are produced in the "lane = query" layout, dS^T feeds
//                   dQ^T += K^T dS^T with K read from LDS by the transposing load.
//   dK/dV kernel -- a workgroup owns 128 key slots and walks query tiles (and the query heads of
//                   its group); S and dP are produced in the "lane = key" layout, P and dS feed
//                   dV^T += dO^T P and dK^T += Q^T dS with dO and Q read by the transposing load.
#include "sa_common.h"
#include "sa_mfma.h"

namespace sa {
namespace {

constexpr int BM = 128;  // stationary slots per workgroup
constexpr int BN = 64;   // streamed slots per tile
constexpr int NT = 256;

template <int D>
struct Cfg {
  static constexpr int STR = D + 8;     // bf16 per LDS row (+16 B pad)
  static constexpr int VPR = D / 8;     // 16-byte vectors per row
  static constexpr int RPP = NT / VPR;
  static constexpr int NV = BN / RPP;
  static constexpr int WRPP = 64 / VPR;
  static constexpr int TILE_BYTES = BN * STR * 2;
  static constexpr int LDS_BYTES = 2 * TILE_BYTES + 3 * BN * 4;
  static_assert(4 * 32 * STR * 2 <= 2 * TILE_BYTES, "per-wave staging must fit in the two tiles");
};

// Stage 32 rows (slots s0 .. s0+31, clamped to n-1) of a [n, D] head through this wave's LDS area
// and return them as MFMA B operands: lane (g2, c32) gets row c32, elements 16kk + 8*g2 .. +7.
template <int D>
__device__ __forceinline__ void load_stationary(const bf16_t* __restrict__ head, const int32_t* __restrict__ perm,
                                                int s0, int n, bf16_t* stage, int lane, bf16x8* frag) {
  using C = Cfg<D>;
  const int chunk16 = lane % C::VPR;
#pragma unroll
  for (int pass = 0; pass < 32 / C::WRPP; ++pass) {
    const int row = pass * C::WRPP + lane / C::VPR;
    const int src = slot_to_orig(perm, min(s0 + row, n - 1));
    const u32x4 v = *reinterpret_cast<const u32x4*>(head + (size_t)src * D + chunk16 * 8);
    *reinterpret_cast<u32x4*>(stage + row * C::STR + chunk16 * 8) = v;
  }
  __syncthreads();
  const int g2 = lane >> 5, c32 = lane & 31;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk)
    frag[kk] = *reinterpret_cast<const bf16x8*>(stage + c32 * C::STR + 16 * kk + 8 * g2);
  __syncthreads();
}

// Write a wave's transposed accumulators (lane = row c32 of the output, 4 consecutive values along
// d per accumulator quad) as 32 bf16 rows to their original positions.  `accumulate` first adds what
// the rows already hold, in fp32, so the sum is rounded once.
template <int D>
__device__ __forceinline__ void store_rows(f32x16* acc, float mul, bf16_t* stage, bf16_t* out_head,
                                           const int32_t* perm, int s0, int n, int lane, int accumulate) {
  using C = Cfg<D>;
  const int g2 = lane >> 5, c32 = lane & 31;
  const bf16_t* mine = out_head + (size_t)slot_to_orig(perm, min(s0 + c32, n - 1)) * D;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int mq = 0; mq < 4; ++mq) {
      float v0 = acc[db][4 * mq + 0] * mul, v1 = acc[db][4 * mq + 1] * mul;
      float v2 = acc[db][4 * mq + 2] * mul, v3 = acc[db][4 * mq + 3] * mul;
      if (accumulate) {
        const u32x2 o = *reinterpret_cast<const u32x2*>(mine + 32 * db + 8 * mq + 4 * g2);
        v0 += bf16lo(o[0]); v1 += bf16hi(o[0]);
        v2 += bf16lo(o[1]); v3 += bf16hi(o[1]);
      }
      u32x2 w;
      w[0] = pack_bf16(v0, v1);
      w[1] = pack_bf16(v2, v3);
      *reinterpret_cast<u32x2*>(stage + c32 * C::STR + 32 * db + 8 * mq + 4 * g2) = w;
    }
  __syncthreads();
  const int chunk16 = lane % C::VPR;
#pragma unroll
  for (int pass = 0; pass < 32 / C::WRPP; ++pass) {
    const int row = pass * C::WRPP + lane / C::VPR;
    if (s0 + row < n) {
      const size_t eoff = (size_t)slot_to_orig(perm, s0 + row) * D + chunk16 * 8;
      *reinterpret_cast<u32x4*>(out_head + eoff) = *reinterpret_cast<const u32x4*>(stage + row * C::STR + chunk16 * 8);
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------ dQ
template <int D>
__global__ __launch_bounds__(NT, D == 128 ? 1 : 2) void bwd_dq_mfma_bf16_kernel(const Pass p, const int num_qt, const long total_work) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem);
  bf16_t* Vs = reinterpret_cast<bf16_t*>(smem + C::TILE_BYTES);
  int* pk_lds = reinterpret_cast<int*>(smem + 2 * C::TILE_BYTES);

  const long work = xcd_work_index(total_work);
  if (work < 0) return;
  const int hg = (int)(work % p.g);
  long rest = work / p.g;
  const int qt = (int)(rest % num_qt);
  rest /= num_qt;
  const int hk = (int)(rest % p.Hkv);
  const int b = (int)(rest / p.Hkv);
  const int hq = hk * p.g + hg;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g2 = lane >> 5, c32 = lane & 31;
  const int n = p.n, L = p.win.L, R = p.win.R;
  const bool circular = p.win.circular != 0, causal = p.causal != 0;
  const int32_t* __restrict__ perm =
      p.perm ? p.perm + (size_t)perm_slice_index(p.perm_B, p.perm_H, b, hq) * n : nullptr;
  const size_t head_row0 = ((size_t)b * p.Hq + hq) * n;
  const bf16_t* __restrict__ Qh = reinterpret_cast<const bf16_t*>(p.Q) + head_row0 * D;
  const bf16_t* __restrict__ dOh = reinterpret_cast<const bf16_t*>(p.dO) + head_row0 * D;
  const bf16_t* __restrict__ Kh = reinterpret_cast<const bf16_t*>(p.K) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  const bf16_t* __restrict__ Vh = reinterpret_cast<const bf16_t*>(p.V) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;

  const int p0 = qt * BM;
  const int q_last = min(p0 + BM - 1, n - 1);
  const int s_w0 = p0 + 32 * wave;
  const int s = s_w0 + c32;
  const int orig_q = slot_to_orig(perm, min(s, n - 1));
  const float lse2 = p.lse_in[head_row0 + orig_q] * kLog2e;
  const float Dq = p.Dsum[head_row0 + orig_q];

  int t_lo = p0 - L, t_hi = q_last + R;
  if (!circular) {
    t_lo = max(t_lo, 0);
    t_hi = min(t_hi, n - 1);
  }
  const int ntiles = (t_hi - t_lo + BN) / BN;

  bf16_t* stage = reinterpret_cast<bf16_t*>(smem) + wave * 32 * C::STR;
  bf16x8 qf[D / 16], gf[D / 16];
  load_stationary<D>(Qh, perm, s_w0, n, stage, lane, qf);
  load_stationary<D>(dOh, perm, s_w0, n, stage, lane, gf);

  const int ld_row = tid / C::VPR, ld_chunk = tid % C::VPR;
  int idx[C::NV];
  int pk_next = 0;
  auto load_idx = [&](int tile) {
    const int t0 = t_lo + tile * BN;
#pragma unroll
    for (int v = 0; v < C::NV; ++v) {
      const int t = min(t0 + v * C::RPP + ld_row, t_hi);
      idx[v] = slot_to_orig(perm, wrap_slot(t, n));
    }
    if (tid < BN) pk_next = slot_to_orig(perm, wrap_slot(min(t0 + tid, t_hi), n));
  };
  u32x4 kreg[C::NV], vreg[C::NV];
  auto load_rows = [&]() {
#pragma unroll
    for (int v = 0; v < C::NV; ++v) {
      kreg[v] = *reinterpret_cast<const u32x4*>(Kh + (size_t)idx[v] * D + ld_chunk * 8);
      vreg[v] = *reinterpret_cast<const u32x4*>(Vh + (size_t)idx[v] * D + ld_chunk * 8);
    }
  };
  load_idx(0);
  load_rows();
  int pk_cur = pk_next;
  if (ntiles > 1) load_idx(1);

  const int Ll = circular ? L : min(L, max(s, 0));
  const int Rl = circular ? R : min(R, max(n - 1 - s, 0));
  const unsigned LRl = (unsigned)(Ll + Rl);
  const float cs = p.scale * kLog2e;

  f32x16 dqacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;

  for (int tile = 0; tile < ntiles; ++tile) {
    __syncthreads();
#pragma unroll
    for (int v = 0; v < C::NV; ++v) {
      const int row = v * C::RPP + ld_row;
      *reinterpret_cast<u32x4*>(Ks + row * C::STR + ld_chunk * 8) = kreg[v];
      *reinterpret_cast<u32x4*>(Vs + row * C::STR + ld_chunk * 8) = vreg[v];
    }
    if (tid < BN) pk_lds[tid] = pk_cur;
    __syncthreads();
    if (tile + 1 < ntiles) {
      load_rows();
      pk_cur = pk_next;
      if (tile + 2 < ntiles) load_idx(tile + 2);
    }
    const int t0 = t_lo + tile * BN;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int tb0 = t0 + 32 * kb;
      const int dmax = tb0 + 31 - s_w0, dmin = tb0 - (s_w0 + 31);
      const bool act = !(dmax < -L || dmin > R) && tb0 <= t_hi;
      const bool inside = dmin >= -L && dmax <= R && tb0 + 31 <= t_hi && s_w0 + 31 <= q_last;
      if (!act) continue;
      f32x16 sacc, dpacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 ka = *reinterpret_cast<const bf16x8*>(Ks + (32 * kb + c32) * C::STR + 16 * kk + 8 * g2);
        sacc = mfma_bf16(ka, qf[kk], sacc);    // S^T = K Q^T
        const bf16x8 va = *reinterpret_cast<const bf16x8*>(Vs + (32 * kb + c32) * C::STR + 16 * kk + 8 * g2);
        dpacc = mfma_bf16(va, gf[kk], dpacc);  // dP^T = V dO^T
      }
      if (causal) {
#pragma unroll
        for (int mq = 0; mq < 4; ++mq) {
          const int4 pk = *reinterpret_cast<const int4*>(pk_lds + 32 * kb + 8 * mq + 4 * g2);
          if (pk.x > orig_q) sacc[4 * mq + 0] = -INFINITY;
          if (pk.y > orig_q) sacc[4 * mq + 1] = -INFINITY;
          if (pk.z > orig_q) sacc[4 * mq + 2] = -INFINITY;
          if (pk.w > orig_q) sacc[4 * mq + 3] = -INFINITY;
        }
      }
      if (!inside) {
        const int base = tb0 + 4 * g2 - s + Ll;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const unsigned u = (unsigned)(base + 8 * (i / 4) + (i % 4));
          if (u > LRl) sacc[i] = -INFINITY;
        }
      }
      float ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pe = __builtin_amdgcn_exp2f(fmaf(sacc[i], cs, -lse2));
        ds[i] = pe * (dpacc[i] - Dq);
      }
      const bf16x8 dsf0 = pack_b_operand(ds), dsf1 = pack_b_operand(ds + 8);
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {  // dQ^T += K^T dS^T
        dqacc[db] = mfma_bf16(lds_read_transposed_a(Ks, C::STR, 32 * kb, 32 * db, lane), dsf0, dqacc[db]);
        dqacc[db] = mfma_bf16(lds_read_transposed_a(Ks, C::STR, 32 * kb + 16, 32 * db, lane), dsf1, dqacc[db]);
      }
    }
  }
  __syncthreads();
  store_rows<D>(dqacc, p.scale, stage, reinterpret_cast<bf16_t*>(p.dQ) + head_row0 * D, perm, s_w0, n, lane, p.accumulate);
}

// --------------------------------------------------------------------------------------- dK, dV
template <int D>
__global__ __launch_bounds__(NT, D == 128 ? 1 : 2) void bwd_dkv_mfma_bf16_kernel(const Pass p, const int num_kt, const long total_work) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];
  bf16_t* Qs = reinterpret_cast<bf16_t*>(smem);
  bf16_t* Gs = reinterpret_cast<bf16_t*>(smem + C::TILE_BYTES);
  int* pq_lds = reinterpret_cast<int*>(smem + 2 * C::TILE_BYTES);
  float* lse_lds = reinterpret_cast<float*>(smem + 2 * C::TILE_BYTES + BN * 4);
  float* dd_lds = reinterpret_cast<float*>(smem + 2 * C::TILE_BYTES + 2 * BN * 4);

  const long work = xcd_work_index(total_work);
  if (work < 0) return;
  const int kt = (int)(work % num_kt);
  long rest = work / num_kt;
  const int hk = (int)(rest % p.Hkv);
  const int b = (int)(rest / p.Hkv);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g2 = lane >> 5, c32 = lane & 31;
  const int n = p.n, L = p.win.L, R = p.win.R;
  const bool circular = p.win.circular != 0, causal = p.causal != 0;
  const bf16_t* __restrict__ Kh = reinterpret_cast<const bf16_t*>(p.K) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  const bf16_t* __restrict__ Vh = reinterpret_cast<const bf16_t*>(p.V) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;

  const int t0w = kt * BM;
  const int t_last = min(t0w + BM - 1, n - 1);
  const int t_w0 = t0w + 32 * wave;
  const int t = t_w0 + c32;  // this lane's key slot (column of S)

  // query-slot range of the workgroup: s in [t - R, t + L]
  int s_lo = t0w - R, s_hi = t_last + L;
  if (!circular) {
    s_lo = max(s_lo, 0);
    s_hi = min(s_hi, n - 1);
  }
  const int ntiles = (s_hi - s_lo + BN) / BN;
  // per-lane bounds: query s sees this key iff smin <= s <= smax
  const int smin = circular ? t - R : max(t - R, 0);
  const int smax = circular ? t + L : min(t + L, n - 1);
  const unsigned srange = (unsigned)max(smax - smin, 0);
  const float cs = p.scale * kLog2e;

  bf16_t* stage = reinterpret_cast<bf16_t*>(smem) + wave * 32 * C::STR;
  f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[db][i] = 0.f; dvacc[db][i] = 0.f; }

  const int32_t* perm = nullptr;
  const int hg_begin = p.hq_only >= 0 ? p.hq_only : 0;
  const int hg_end = p.hq_only >= 0 ? p.hq_only + 1 : p.g;
  bf16x8 kf[D / 16], vf[D / 16];
  int orig_k = 0;
  for (int hg = hg_begin; hg < hg_end; ++hg) {
    const int hq = hk * p.g + hg;
    const int32_t* __restrict__ perm_h =
        p.perm ? p.perm + (size_t)perm_slice_index(p.perm_B, p.perm_H, b, hq) * n : nullptr;
    if (hg == hg_begin || perm_h != perm) {
      // (re)load the stationary K and V rows; with one permutation per group this happens once
      perm = perm_h;
      __syncthreads();
      load_stationary<D>(Kh, perm, t_w0, n, stage, lane, kf);
      load_stationary<D>(Vh, perm, t_w0, n, stage, lane, vf);
      orig_k = slot_to_orig(perm, min(t, n - 1));
    }
    const size_t head_row0 = ((size_t)b * p.Hq + hq) * n;
    const bf16_t* __restrict__ Qh = reinterpret_cast<const bf16_t*>(p.Q) + head_row0 * D;
    const bf16_t* __restrict__ dOh = reinterpret_cast<const bf16_t*>(p.dO) + head_row0 * D;
    const float* __restrict__ lse_h = p.lse_in + head_row0;
    const float* __restrict__ dd_h = p.Dsum + head_row0;

    const int ld_row = tid / C::VPR, ld_chunk = tid % C::VPR;
    int idx[C::NV];
    int pq_next = 0;
    auto load_idx = [&](int tile) {
      const int s0 = s_lo + tile * BN;
#pragma unroll
      for (int v = 0; v < C::NV; ++v) {
        const int sq = min(s0 + v * C::RPP + ld_row, s_hi);
        idx[v] = slot_to_orig(perm, wrap_slot(sq, n));
      }
      if (tid < BN) pq_next = slot_to_orig(perm, wrap_slot(min(s0 + tid, s_hi), n));
    };
    u32x4 qreg[C::NV], greg[C::NV];
    float lse_reg = 0.f, dd_reg = 0.f;
    int pq_cur = 0;
    auto load_rows = [&]() {
#pragma unroll
      for (int v = 0; v < C::NV; ++v) {
        qreg[v] = *reinterpret_cast<const u32x4*>(Qh + (size_t)idx[v] * D + ld_chunk * 8);
        greg[v] = *reinterpret_cast<const u32x4*>(dOh + (size_t)idx[v] * D + ld_chunk * 8);
      }
      if (tid < BN) {
        pq_cur = pq_next;
        lse_reg = lse_h[pq_next] * kLog2e;
        dd_reg = dd_h[pq_next];
      }
    };
    load_idx(0);
    load_rows();
    if (ntiles > 1) load_idx(1);

    for (int tile = 0; tile < ntiles; ++tile) {
      __syncthreads();
#pragma unroll
      for (int v = 0; v < C::NV; ++v) {
        const int row = v * C::RPP + ld_row;
        *reinterpret_cast<u32x4*>(Qs + row * C::STR + ld_chunk * 8) = qreg[v];
        *reinterpret_cast<u32x4*>(Gs + row * C::STR + ld_chunk * 8) = greg[v];
      }
      if (tid < BN) {
        pq_lds[tid] = pq_cur;
        lse_lds[tid] = lse_reg;
        dd_lds[tid] = dd_reg;
      }
      __syncthreads();
      if (tile + 1 < ntiles) {
        load_rows();
        if (tile + 2 < ntiles) load_idx(tile + 2);
      }
      const int s0 = s_lo + tile * BN;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int sb0 = s0 + 32 * qb;
        const int dmax = t_w0 + 31 - sb0, dmin = t_w0 - (sb0 + 31);  // range of t - s over the block
        const bool act = !(dmax < -L || dmin > R) && sb0 <= s_hi;
        const bool inside = dmin >= -L && dmax <= R && sb0 + 31 <= s_hi && t_w0 + 31 <= t_last;
        if (!act) continue;
        f32x16 sacc, dpacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(Qs + (32 * qb + c32) * C::STR + 16 * kk + 8 * g2);
          sacc = mfma_bf16(qa, kf[kk], sacc);    // S = Q K^T
          const bf16x8 ga = *reinterpret_cast<const bf16x8*>(Gs + (32 * qb + c32) * C::STR + 16 * kk + 8 * g2);
          dpacc = mfma_bf16(ga, vf[kk], dpacc);  // dP = dO V^T
        }
        // accumulator i is query row 32*qb + 8*(i/4) + 4*g2 + i%4 of the tile, key column = lane
        if (causal) {
#pragma unroll
          for (int mq = 0; mq < 4; ++mq) {
            const int4 pq = *reinterpret_cast<const int4*>(pq_lds + 32 * qb + 8 * mq + 4 * g2);
            if (pq.x < orig_k) sacc[4 * mq + 0] = -INFINITY;
            if (pq.y < orig_k) sacc[4 * mq + 1] = -INFINITY;
            if (pq.z < orig_k) sacc[4 * mq + 2] = -INFINITY;
            if (pq.w < orig_k) sacc[4 * mq + 3] = -INFINITY;
          }
        }
        if (!inside) {
          const int base = sb0 + 4 * g2 - smin;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const unsigned u = (unsigned)(base + 8 * (i / 4) + (i % 4));
            if (u > srange || smax < smin) sacc[i] = -INFINITY;
          }
        }
        float pe[16], ds[16];
#pragma unroll
        for (int mq = 0; mq < 4; ++mq) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_lds + 32 * qb + 8 * mq + 4 * g2);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(dd_lds + 32 * qb + 8 * mq + 4 * g2);
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const int i = 4 * mq + x;
            pe[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], cs, -l4[x]));
            ds[i] = pe[i] * (dpacc[i] - d4[x]);
          }
        }
        const bf16x8 pf0 = pack_b_operand(pe), pf1 = pack_b_operand(pe + 8);
        const bf16x8 dsf0 = pack_b_operand(ds), dsf1 = pack_b_operand(ds + 8);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
          // dV^T += dO^T P,  dK^T += Q^T dS  (contraction over the 32 query rows of the block)
          dvacc[db] = mfma_bf16(lds_read_transposed_a(Gs, C::STR, 32 * qb, 32 * db, lane), pf0, dvacc[db]);
          dvacc[db] = mfma_bf16(lds_read_transposed_a(Gs, C::STR, 32 * qb + 16, 32 * db, lane), pf1, dvacc[db]);
          dkacc[db] = mfma_bf16(lds_read_transposed_a(Qs, C::STR, 32 * qb, 32 * db, lane), dsf0, dkacc[db]);
          dkacc[db] = mfma_bf16(lds_read_transposed_a(Qs, C::STR, 32 * qb + 16, 32 * db, lane), dsf1, dkacc[db]);
        }
      }
    }
  }
  __syncthreads();
  bf16_t* dKh = reinterpret_cast<bf16_t*>(p.dK) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  bf16_t* dVh = reinterpret_cast<bf16_t*>(p.dV) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  store_rows<D>(dkacc, p.scale, stage, dKh, perm, t_w0, n, lane, p.accumulate);
  store_rows<D>(dvacc, 1.f, stage, dVh, perm, t_w0, n, lane, p.accumulate);
}

template <int D>
hipError_t launch_dq_t(const Pass& p, hipStream_t st) {
  const int num_qt = (p.n + BM - 1) / BM;
  const long total = (long)num_qt * p.Hq * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((bwd_dq_mfma_bf16_kernel<D>), dim3((unsigned)blocks), dim3(NT), 0, st, p, num_qt, total);
  return hipGetLastError();
}

template <int D>
hipError_t launch_dkv_t(const Pass& p, hipStream_t st) {
  const int num_kt = (p.n + BM - 1) / BM;
  const long total = (long)num_kt * p.Hkv * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((bwd_dkv_mfma_bf16_kernel<D>), dim3((unsigned)blocks), dim3(NT), 0, st, p, num_kt, total);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_mfma_bf16(const Pass& p, hipStream_t st) {
  if (p.n < 1 || p.B < 1 || p.Hq < 1 || p.Hkv < 1 || p.g * p.Hkv != p.Hq) return hipErrorInvalidValue;
  if (p.win.L < 0 || p.win.R < 0 || p.win.L >= p.n || p.win.R >= p.n) return hipErrorInvalidValue;
  if (p.win.circular && p.win.L + p.win.R + 1 > p.n) return hipErrorInvalidValue;
  if (!p.dO || !p.lse_in || !p.Dsum || !p.dQ || !p.dK || !p.dV) return hipErrorInvalidValue;
  if (!(p.d == 64 || p.d == 128)) return hipErrorNotSupported;
  hipError_t e = p.d == 64 ? launch_dq_t<64>(p, st) : launch_dq_t<128>(p, st);
  if (e != hipSuccess) return e;
  if (p.perm && p.perm_H != 1 && p.g > 1) {
    // every query head of a group has its own slot order: one pass per head, summed in place
    Pass q = p;
    for (int hg = 0; hg < p.g; ++hg) {
      q.hq_only = hg;
      q.accumulate = (hg == 0) ? p.accumulate : 1;
      e = p.d == 64 ? launch_dkv_t<64>(q, st) : launch_dkv_t<128>(q, st);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  return p.d == 64 ? launch_dkv_t<64>(p, st) : launch_dkv_t<128>(p, st);
}

}  // namespace sa
