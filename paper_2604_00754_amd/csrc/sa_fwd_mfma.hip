// bf16 forward of Stochastic Attention on gfx950 matrix cores.
//
// One workgroup (4 wavefronts) owns 128 consecutive PERMUTED slots of one (batch, query head); a
// wavefront owns 32 of them.  The workgroup walks the slots of the window band (Eq. 3) in tiles of
// 64; K and V rows of a tile are read through the index tensor straight from their original
// positions (the permuted copies of Alg. 1 never exist), staged in LDS, and consumed by
//   S^T = K Q^T          (v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q held in registers)
//   mask: window on slot offsets, causal test on original positions (Sec. 3.3, App. B)
//   online softmax (Eq. 1) -- in the S^T layout a lane holds one query column, so row statistics
//   are lane-local up to one exchange with lane^32
//   O^T += V^T P^T       (A = V read from LDS with the transposing ds_read_b64_tr_b16, B = P^T
//                         taken directly from the S^T accumulators)
// The epilogue normalises, transposes through LDS and writes each row to its ORIGINAL position
// (the "undo permute" of Alg. 1), optionally forming the gated sum of Eq. 5 on the way out.
#include "sa_common.h"
#include "sa_mfma.h"

namespace sa {
namespace {

constexpr int BM = 128;  // query slots per workgroup
constexpr int BN = 64;   // key slots per tile
constexpr int NT = 256;  // threads per workgroup

template <int D>
struct Cfg {
  static constexpr int KSTR = D + 8;    // bf16 per K row in LDS: +16 B keeps 16 consecutive rows on distinct banks for b128 reads
  static constexpr int VSTR = D + 32;   // bf16 per V row in LDS: +64 B spreads 4 consecutive rows over the 4 bank quadrants for the transposing read
  static constexpr int VPR = D / 8;     // 16-byte vectors per row
  static constexpr int RPP = NT / VPR;  // tile rows covered by one pass of the workgroup
  static constexpr int NV = BN / RPP;   // vectors per thread per tile (per tensor)
  static constexpr int WRPP = 64 / VPR; // rows covered by one pass of a single wave
  static constexpr int KBYTES = BN * KSTR * 2;
  static constexpr int VBYTES = BN * VSTR * 2;
  static constexpr int QBYTES = 4 * 32 * KSTR * 2;  // per-wave Q / O staging, aliases K|V
  static constexpr int LDS_BYTES = KBYTES + VBYTES + BN * 4;
  static_assert(QBYTES <= KBYTES + VBYTES, "staging must fit in the K|V area");
};

template <int D>
__global__ __launch_bounds__(NT, 2) void fwd_mfma_bf16_kernel(const Pass p, const int num_qt, const long total_work) {
  using C = Cfg<D>;
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem);
  bf16_t* Vs = reinterpret_cast<bf16_t*>(smem + C::KBYTES);
  int* pk_lds = reinterpret_cast<int*>(smem + C::KBYTES + C::VBYTES);

  // work list order: the query heads of a group, then the next query tile -- neighbours share K/V rows
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
  const bf16_t* __restrict__ Qh = reinterpret_cast<const bf16_t*>(p.Q) + ((size_t)b * p.Hq + hq) * n * (size_t)D;
  const bf16_t* __restrict__ Kh = reinterpret_cast<const bf16_t*>(p.K) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  const bf16_t* __restrict__ Vh = reinterpret_cast<const bf16_t*>(p.V) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;

  const int p0 = qt * BM;
  const int q_last = min(p0 + BM - 1, n - 1);
  const int s_w0 = p0 + 32 * wave;  // first query slot of this wave
  const int s = s_w0 + c32;         // this lane's query slot (column of S^T)
  const int orig_q = slot_to_orig(perm, min(s, n - 1));

  // key-slot range of the workgroup, unwrapped
  int t_lo = p0 - L, t_hi = q_last + R;
  if (!circular) {
    t_lo = max(t_lo, 0);
    t_hi = min(t_hi, n - 1);
  }
  const int ntiles = (t_hi - t_lo + BN) / BN;

  // ---- stage this wave's 32 query rows through LDS and keep them as B operands
  bf16_t* Qs = reinterpret_cast<bf16_t*>(smem) + wave * 32 * C::KSTR;
  {
    const int chunk16 = lane % C::VPR;
#pragma unroll
    for (int pass = 0; pass < 32 / C::WRPP; ++pass) {
      const int row = pass * C::WRPP + lane / C::VPR;
      const int src = slot_to_orig(perm, min(s_w0 + row, n - 1));
      const u32x4 v = *reinterpret_cast<const u32x4*>(Qh + (size_t)src * D + chunk16 * 8);
      *reinterpret_cast<u32x4*>(Qs + row * C::KSTR + chunk16 * 8) = v;
    }
  }
  __syncthreads();
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8*>(Qs + c32 * C::KSTR + 16 * kk + 8 * g2);

  // ---- tile loader: thread -> rows (v*RPP + tid/VPR), 16-byte chunk tid%VPR
  const int ld_row = tid / C::VPR, ld_chunk = tid % C::VPR;
  int idx[C::NV];  // original indices of this thread's rows of the tile being fetched next
  int pk_next = 0; // original index of tile row `tid` (threads < BN), for the causal test
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

  // ---- per-lane window constants: key t is visible iff 0 <= t - s + Ll <= LRl (unsigned compare)
  const int Ll = circular ? L : min(L, max(s, 0));
  const int Rl = circular ? R : min(R, max(n - 1 - s, 0));
  const unsigned LRl = (unsigned)(Ll + Rl);

  const float cs = p.scale * kLog2e;  // exp(scale*x) = exp2(cs*x)
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 oacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;

  for (int tile = 0; tile < ntiles; ++tile) {
    __syncthreads();  // everyone is done reading the previous tile (and the Q staging)
#pragma unroll
    for (int v = 0; v < C::NV; ++v) {
      const int row = v * C::RPP + ld_row;
      *reinterpret_cast<u32x4*>(Ks + row * C::KSTR + ld_chunk * 8) = kreg[v];
      *reinterpret_cast<u32x4*>(Vs + row * C::VSTR + ld_chunk * 8) = vreg[v];
    }
    if (tid < BN) pk_lds[tid] = pk_cur;
    __syncthreads();
    if (tile + 1 < ntiles) {  // fetch the next tile while this one is consumed
      load_rows();
      pk_cur = pk_next;
      if (tile + 2 < ntiles) load_idx(tile + 2);
    }

    const int t0 = t_lo + tile * BN;
    bool act[2], inside[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int tb0 = t0 + 32 * kb;
      const int dmax = tb0 + 31 - s_w0, dmin = tb0 - (s_w0 + 31);
      act[kb] = !(dmax < -L || dmin > R) && tb0 <= t_hi;
      inside[kb] = dmin >= -L && dmax <= R && tb0 + 31 <= t_hi && s_w0 + 31 <= q_last;
    }
    if (!act[0] && !act[1]) continue;

    // ---- S^T = K Q^T for the active 32-slot blocks
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      if (act[kb]) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(Ks + (32 * kb + c32) * C::KSTR + 16 * kk + 8 * g2);
          sacc[kb] = mfma_bf16(a, qf[kk], sacc[kb]);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kb][i] = -INFINITY;
      }
    }

    // ---- mask.  Accumulator i of block kb is key row 32*kb + 8*(i/4) + 4*g2 + i%4 of the tile.
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      if (!act[kb]) continue;
      if (causal) {
#pragma unroll
        for (int mq = 0; mq < 4; ++mq) {
          const int4 pk = *reinterpret_cast<const int4*>(pk_lds + 32 * kb + 8 * mq + 4 * g2);
          if (pk.x > orig_q) sacc[kb][4 * mq + 0] = -INFINITY;
          if (pk.y > orig_q) sacc[kb][4 * mq + 1] = -INFINITY;
          if (pk.z > orig_q) sacc[kb][4 * mq + 2] = -INFINITY;
          if (pk.w > orig_q) sacc[kb][4 * mq + 3] = -INFINITY;
        }
      }
      if (!inside[kb]) {
        const int base = t0 + 32 * kb + 4 * g2 - s + Ll;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const unsigned u = (unsigned)(base + 8 * (i / 4) + (i % 4));
          if (u > LRl) sacc[kb][i] = -INFINITY;
        }
      }
    }

    // ---- online softmax (Eq. 1) on the lane's query column
    float mx = sacc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    if (__any(m_new > m_run)) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_safe) * cs);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
    }
    m_run = m_new;
    const float mc = m_safe * cs;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      if (!act[kb]) continue;
      float pe[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pe[i] = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], cs, -mc));
        l_run += pe[i];
      }
      pf[kb][0] = pack_b_operand(pe);
      pf[kb][1] = pack_b_operand(pe + 8);
    }

    // ---- O^T += V^T P^T.  MFMA step (kb,c) contracts the 16 tile rows 32kb+16c+{0..3,8..11}+4*g2
    // (+4 for the second half of the lane's 8 values); the transposing read fetches exactly those.
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      if (!act[kb]) continue;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
          oacc[db] = mfma_bf16(lds_read_transposed_a(Vs, C::VSTR, 32 * kb + 16 * c, 32 * db, lane), pf[kb][c], oacc[db]);
    }
  }

  // ---- epilogue: normalise, transpose through LDS, scatter rows to their original positions
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv_l = 1.f / l_tot;
  __syncthreads();  // all waves are done with the last tile before the staging area is reused
  bf16_t* Os = reinterpret_cast<bf16_t*>(smem) + wave * 32 * C::KSTR;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int mq = 0; mq < 4; ++mq) {
      u32x2 w;
      w[0] = pack_bf16(oacc[db][4 * mq + 0] * inv_l, oacc[db][4 * mq + 1] * inv_l);
      w[1] = pack_bf16(oacc[db][4 * mq + 2] * inv_l, oacc[db][4 * mq + 3] * inv_l);
      *reinterpret_cast<u32x2*>(Os + c32 * C::KSTR + 32 * db + 8 * mq + 4 * g2) = w;
    }
  const size_t head_row0 = ((size_t)b * p.Hq + hq) * n;
  if (p.LSE && g2 == 0 && s < n) p.LSE[head_row0 + orig_q] = m_run * p.scale + __logf(l_tot);
  __syncthreads();
  {
    const int chunk16 = lane % C::VPR;
#pragma unroll
    for (int pass = 0; pass < 32 / C::WRPP; ++pass) {
      const int row = pass * C::WRPP + lane / C::VPR;
      if (s_w0 + row >= n) continue;
      const size_t orow = head_row0 + slot_to_orig(perm, s_w0 + row);
      const u32x4 y = *reinterpret_cast<const u32x4*>(Os + row * C::KSTR + chunk16 * 8);
      const size_t eoff = orow * D + chunk16 * 8;
      if (p.Y) *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(p.Y) + eoff) = y;
      if (p.gate_mode) {
        // Eq. 5: Y = sig(gamma_this) * Y_this + sig(gamma_other) * Y_other
        const u32x4 o = *reinterpret_cast<const u32x4*>(reinterpret_cast<const bf16_t*>(p.Y_other) + eoff);
        u32x4 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const size_t g0 = p.gate_per_dim ? eoff + 2 * e : orow;
          const size_t g1 = p.gate_per_dim ? eoff + 2 * e + 1 : orow;
          const float ga0 = sigmoidf_exact(load_gate(p.gate_this, g0, p.gate_f32));
          const float ga1 = sigmoidf_exact(load_gate(p.gate_this, g1, p.gate_f32));
          const float gb0 = sigmoidf_exact(load_gate(p.gate_other, g0, p.gate_f32));
          const float gb1 = sigmoidf_exact(load_gate(p.gate_other, g1, p.gate_f32));
          r[e] = pack_bf16(ga0 * bf16lo(y[e]) + gb0 * bf16lo(o[e]), ga1 * bf16hi(y[e]) + gb1 * bf16hi(o[e]));
        }
        *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(p.Yout) + eoff) = r;
      }
    }
  }
}

template <int D>
hipError_t launch_t(const Pass& p, hipStream_t st) {
  const int num_qt = (p.n + BM - 1) / BM;
  const long total = (long)num_qt * p.Hq * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((fwd_mfma_bf16_kernel<D>), dim3((unsigned)blocks), dim3(NT), 0, st, p, num_qt, total);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_mfma_bf16(const Pass& p, hipStream_t st) {
  // geometry the kernel relies on
  if (p.n < 1 || p.B < 1 || p.Hq < 1 || p.Hkv < 1 || p.g * p.Hkv != p.Hq) return hipErrorInvalidValue;
  if (p.win.L < 0 || p.win.R < 0 || p.win.L >= p.n || p.win.R >= p.n) return hipErrorInvalidValue;
  if (p.win.circular && p.win.L + p.win.R + 1 > p.n) return hipErrorInvalidValue;
  if (p.gate_mode && (!p.gate_this || !p.gate_other || !p.Y_other || !p.Yout)) return hipErrorInvalidValue;
  if (p.d == 64) return launch_t<64>(p, st);
  if (p.d == 128) return launch_t<128>(p, st);
  return hipErrorNotSupported;
}

}  // namespace sa
