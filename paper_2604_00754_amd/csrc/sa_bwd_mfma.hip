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
//                   dQ^T += K^T dS^T with K read from LDS by the transposing load.  Given the forward's
//                   output rows it also forms D for its queries (it holds their dO rows anyway) and
//                   leaves D for the other kernel, so the ungated call has no separate row-sum pass.
//   dK/dV kernel -- a workgroup owns 128 key slots and walks query tiles (and the query heads of
//                   its group); S and dP are produced in the "lane = key" layout, P and dS feed
//                   dV^T += dO^T P and dK^T += Q^T dS with dO and Q read by the transposing load.
#include "sa_common.h"
#include "sa_mfma.h"

namespace sa {
namespace {

// Waves per SIMD the kernels are compiled for (register budget 512 / waves per lane), and the streamed slots per
// tile of the dK/dV kernel.  At d = 128 the dK/dV kernel holds 128 accumulators and 64 stationary operand
// registers per lane: one wave per SIMD.
constexpr int DQ64_WAVES = 3, DQ128_WAVES = 2, DKV64_WAVES = 2, DKV128_WAVES = 1;
constexpr int DKV64_BN = 128, DKV128_BN = 64;
constexpr int BM = 128;  // stationary slots per workgroup
constexpr int NT = 256;

// How the causal conjunct (original position of the key <= that of the query) is applied:
//   CAUSAL_I32 -- compare 32-bit original positions on the fp32 scores (any n),
//   CAUSAL_I16 -- n <= 65535: biased 16-bit positions, kept in LDS in accumulator order, turn into an
//                 AND mask on the bf16 pairs that feed the next product (three 2-wide instructions
//                 per pair instead of two compares and two selects).
enum { CAUSAL_NONE = 0, CAUSAL_I32 = 1, CAUSAL_I16 = 2 };

typedef short s16x2 __attribute__((ext_vector_type(2)));

template <int D, int BN_>
struct Cfg {
  static constexpr int BN = BN_;         // streamed slots per tile
  static constexpr int STR = D + 8;      // bf16 per row of the wave-private staging areas (+16 B pad)
  static constexpr int VPR = D / 8;      // 16-byte vectors per row
  static constexpr int RPP = NT / VPR;   // streamed rows the workgroup moves with one instruction per wave
  static constexpr int NV = BN / RPP;    // such instructions per tile and operand
  static constexpr int WRPP = 64 / VPR;  // rows one wave moves per pass
  static constexpr int SP = 32 / WRPP;   // passes for a wave's 32 stationary rows
  static constexpr int TILE_BYTES = BN * D * 2;           // one streamed operand tile: rows unpadded, chunks swizzled
  static constexpr int BUF_BYTES = 2 * TILE_BYTES;        // the two streamed operands of a tile
  static constexpr int STAGE_BYTES = 4 * 32 * STR * 2;    // 32 staged rows of each of the 4 waves
  // buffer 0 | buffer 1, which the staging area shares (it is used before tile 1 is requested and after
  // the last tile) | per-slot values of two tiles
  static constexpr int AREA_BYTES = BUF_BYTES + (BUF_BYTES > STAGE_BYTES ? BUF_BYTES : STAGE_BYTES);
  static constexpr int SLOT_BYTES = 3 * BN * 4;
  static constexpr int LDS_BYTES = AREA_BYTES + 2 * SLOT_BYTES;
  static_assert(BN <= NT && BN % 32 == 0 && NV >= 1, "one thread per streamed slot for the per-slot values");
};

// Accumulator i = 4*mq + x of lane group g2 holds tile row 32*kb + 8*mq + 4*g2 + x.  Position of tile
// row r in "accumulator order": the 16 rows of one (kb, g2) are contiguous, in the order of i.
__device__ __forceinline__ int acc_order_pos(int r) {
  return (r & ~31) | (((r >> 2) & 1) << 4) | (((r >> 3) & 3) << 2) | (r & 3);
}

// The 32 stationary rows of a wave (slots s0 .. s0+31, clamped to n-1) reach the MFMA B-operand layout
// through a wave-private LDS area, in steps, so that a kernel can put every index load, then every row
// load of its prologue in flight before it waits for any of them:
//   stationary_src  -- original positions of the rows this lane moves,
//   stationary_rows -- the lane's 16-byte pieces of those rows,
//   stationary_put / stationary_get -- through LDS: lane (g2, c32) gets row c32, elements
//   16kk + 8*g2 .. +7.
template <class C>
__device__ __forceinline__ void stationary_src(const int32_t* __restrict__ perm, int s0, int n, int lane, int* src) {
#pragma unroll
  for (int pass = 0; pass < C::SP; ++pass)
    src[pass] = slot_to_orig(perm, min(s0 + pass * C::WRPP + lane / C::VPR, n - 1));
}

template <class C, int D>
__device__ __forceinline__ void stationary_rows(const bf16_t* __restrict__ head, const int* src, int lane, u32x4* rows) {
#pragma unroll
  for (int pass = 0; pass < C::SP; ++pass)
    rows[pass] = *reinterpret_cast<const u32x4*>(head + (size_t)src[pass] * D + (lane % C::VPR) * 8);
}

template <class C>
__device__ __forceinline__ void stationary_put(bf16_t* stage, int lane, const u32x4* rows) {
#pragma unroll
  for (int pass = 0; pass < C::SP; ++pass)
    *reinterpret_cast<u32x4*>(stage + (pass * C::WRPP + lane / C::VPR) * C::STR + (lane % C::VPR) * 8) = rows[pass];
}

template <class C, int D>
__device__ __forceinline__ void stationary_get(const bf16_t* stage, int lane, bf16x8* frag) {
  const int g2 = lane >> 5, c32 = lane & 31;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk)
    frag[kk] = *reinterpret_cast<const bf16x8*>(stage + c32 * C::STR + 16 * kk + 8 * g2);
}

// Write a wave's transposed accumulators (lane = row c32 of the output, 4 consecutive values along
// d per accumulator quad) as 32 bf16 rows to their original positions: src[pass] for the rows this
// lane moves (as stationary_src gave them).  `accumulate`
// first adds what the rows already hold (the other branch's gradient, stored as bf16) in fp32 and rounds
// the sum: two roundings in all, one per branch.  The staging area is private to the wave.
// trow != nullptr: the rows are first turned back by the angle of their position (the transpose of RoPE).
template <class C, int D>
__device__ __forceinline__ void store_rows(f32x16* acc, float mul, bf16_t* stage, bf16_t* out_head, const int* src,
                                           int orig_mine, int s0, int n, int lane, int accumulate,
                                           const float2* trow = nullptr, int interleaved = 0) {
  const int g2 = lane >> 5, c32 = lane & 31;
  if (trow) rope_transpose_accumulators<D>(acc, trow, g2, interleaved);
  if (accumulate) {
    // what the rows hold comes in as whole rows, the way they leave (in the accumulator layout a lane would ask
    // memory for 8-byte pieces of 32 rows per instruction), and waits in the staging area for the sums
    u32x4 old[C::SP];
#pragma unroll
    for (int pass = 0; pass < C::SP; ++pass)
      old[pass] = *reinterpret_cast<const u32x4*>(out_head + (size_t)src[pass] * D + (lane % C::VPR) * 8);
#pragma unroll
    for (int pass = 0; pass < C::SP; ++pass)
      *reinterpret_cast<u32x4*>(stage + (pass * C::WRPP + lane / C::VPR) * C::STR + (lane % C::VPR) * 8) = old[pass];
    wave_lds_sync();
  }
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int mq = 0; mq < 4; ++mq) {
      float v0 = acc[db][4 * mq + 0] * mul, v1 = acc[db][4 * mq + 1] * mul;
      float v2 = acc[db][4 * mq + 2] * mul, v3 = acc[db][4 * mq + 3] * mul;
      if (accumulate) {
        const u32x2 o = *reinterpret_cast<const u32x2*>(stage + c32 * C::STR + 32 * db + 8 * mq + 4 * g2);
        v0 += bf16lo(o[0]); v1 += bf16hi(o[0]);
        v2 += bf16lo(o[1]); v3 += bf16hi(o[1]);
      }
      u32x2 w;
      w[0] = pack_bf16(v0, v1);
      w[1] = pack_bf16(v2, v3);
      *reinterpret_cast<u32x2*>(stage + c32 * C::STR + 32 * db + 8 * mq + 4 * g2) = w;
    }
  wave_lds_sync();
  const int chunk16 = lane % C::VPR;
#pragma unroll
  for (int pass = 0; pass < C::SP; ++pass) {
    const int row = pass * C::WRPP + lane / C::VPR;
    if (s0 + row < n) {
      const size_t eoff = (size_t)src[pass] * D + chunk16 * 8;
      __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(stage + row * C::STR + chunk16 * 8),
                                  reinterpret_cast<u32x4*>(out_head + eoff));
    }
  }
  wave_lds_sync();
}

// ------------------------------------------------------------------------------------------ dQ
template <int D, int CAUSAL>
__global__ __launch_bounds__(NT, D == 128 ? DQ128_WAVES : DQ64_WAVES) void bwd_dq_mfma_bf16_kernel(const Pass p, const int num_qt, const long total_work,
                                                                                            const int hshift) {
  using C = Cfg<D, 64>;
  constexpr int BN = C::BN;
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

  // 1 << hshift query heads of a KV group share the workgroup (as in the forward: the same 32 slots of
  // up to four heads that read K/V through one permutation, one head per wave); 0: four 32-slot blocks of
  // one head.  Work list order: the head sets of a KV group, then the next query tile.
  const long work = xcd_work_index(total_work);
  if (work < 0) return;
  const int sets = p.g >> hshift;
  const int hset = (int)(work % sets);
  long rest = work / sets;
  const int qt = (int)(rest % num_qt);
  rest /= num_qt;
  const int hk = (int)(rest % p.Hkv);
  const int b = (int)(rest / p.Hkv);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hq = hk * p.g + (hset << hshift) + (wave & ((1 << hshift) - 1));  // this wave's query head
  const int bm = BM >> hshift;                                               // query slots of the workgroup
  const int g2 = lane >> 5, c32 = lane & 31;
  const int n = p.n, L = p.win.L, R = p.win.R;
  const bool circular = p.win.circular != 0;
  const int32_t* __restrict__ perm =
      p.perm ? p.perm + (size_t)perm_slice_index(p.perm_B, p.perm_H, b, hq) * n : nullptr;
  const size_t head_row0 = ((size_t)b * p.Hq + hq) * n;
  const bf16_t* __restrict__ Qh = reinterpret_cast<const bf16_t*>(p.Q) + head_row0 * D;
  const bf16_t* __restrict__ dOh = reinterpret_cast<const bf16_t*>(p.dO) + head_row0 * D;
  const bf16_t* __restrict__ Kh = reinterpret_cast<const bf16_t*>(p.K) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  const bf16_t* __restrict__ Vh = reinterpret_cast<const bf16_t*>(p.V) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;

  const int p0 = qt * bm;
  const int q_last = min(p0 + bm - 1, n - 1);
  const int s_w0 = p0 + 32 * (wave >> hshift);
  const int s = s_w0 + c32;

  int t_lo = p0 - L, t_hi = q_last + R;
  if (!circular) {
    t_lo = max(t_lo, 0);
    t_hi = min(t_hi, n - 1);
  }
  const int ntiles = (t_hi - t_lo + BN) / BN;

  // streamed tiles: K | V rows of 64 key slots, fetched through the index tensor by direct global-to-LDS
  // loads one tile ahead (double buffered, one barrier per tile).  Instruction v of a wave fills rows
  // v*RPP + wave*WRPP .. of the tile; the lane delivers physical chunk lane % VPR of its row.
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const int ld_row = tid / C::VPR;
  const uint32_t ld_chunk_off = (uint32_t)((((tid % C::VPR)) ^ swz<D>(ld_row)) * 16);
  const int pk_pos = acc_order_pos(tid & (BN - 1));
  int idx[C::NV];
  int pk_next = 0;
  auto load_idx = [&](int tile) {
    const int t0 = t_lo + tile * BN;
#pragma unroll
    for (int v = 0; v < C::NV; ++v) {
      const int t = min(t0 + v * C::RPP + ld_row, t_hi);
      idx[v] = slot_to_orig(perm, wrap_slot(t, n));
    }
    if (CAUSAL != CAUSAL_NONE && tid < BN) pk_next = slot_to_orig(perm, wrap_slot(min(t0 + tid, t_hi), n));
  };
  // requests the tile whose indices load_idx fetched last, and publishes its causal positions
  auto request_tile = [&](const int buf) {
#pragma unroll
    for (int v = 0; v < C::NV; ++v) {
      const uint32_t goff = (uint32_t)idx[v] * (uint32_t)(D * 2) + ld_chunk_off;
      const uint32_t dst = lds0 + buf * C::BUF_BYTES + (v * C::RPP + wave * C::WRPP) * (D * 2);
      load_to_lds_16(Kh, goff, dst);
      load_to_lds_16(Vh, goff, dst + C::TILE_BYTES);
    }
    if (CAUSAL == CAUSAL_I32 && tid < BN) reinterpret_cast<int*>(smem + C::AREA_BYTES + buf * C::SLOT_BYTES)[tid] = pk_next;
    if (CAUSAL == CAUSAL_I16 && tid < BN)
      reinterpret_cast<short*>(smem + C::AREA_BYTES + buf * C::SLOT_BYTES)[pk_pos] = (short)(pk_next - 32768);
  };

  // prologue: every index, then every row (first K/V tile, stationary Q and dO), then the staging
  int st_src[C::SP];
  stationary_src<C>(perm, s_w0, n, lane, st_src);
  const int orig_q = slot_to_orig(perm, min(s, n - 1));
  load_idx(0);
  bf16x8 qf[D / 16], gf[D / 16];
  float Dq = 0.f;
  {
    u32x4 qrow[C::SP], grow[C::SP], orow[C::SP];
    stationary_rows<C, D>(Qh, st_src, lane, qrow);
    stationary_rows<C, D>(dOh, st_src, lane, grow);
    if (p.O_rows) stationary_rows<C, D>(reinterpret_cast<const bf16_t*>(p.O_rows) + head_row0 * D, st_src, lane, orow);
    request_tile(0);
    if (ntiles > 1) load_idx(1);
    bf16_t* stage = reinterpret_cast<bf16_t*>(smem + C::BUF_BYTES) + wave * 32 * C::STR;  // buffer 1 is still free
    stationary_put<C>(stage, lane, qrow);
    wave_lds_sync();
    stationary_get<C, D>(stage, lane, qf);
    wave_lds_sync();
    stationary_put<C>(stage, lane, grow);
    wave_lds_sync();
    stationary_get<C, D>(stage, lane, gf);
    if (p.O_rows) {
      // D = rowsum(dO o O) of the lane's query row, from the rows this wave holds anyway: the output rows take the
      // same way as Q and dO, each lane sums its half of the row and the two halves are added
      bf16x8 of[D / 16];
      wave_lds_sync();
      stationary_put<C>(stage, lane, orow);
      wave_lds_sync();
      stationary_get<C, D>(stage, lane, of);
      float part = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const u32x4 gw = __builtin_bit_cast(u32x4, gf[kk]), ow = __builtin_bit_cast(u32x4, of[kk]);
#pragma unroll
        for (int e = 0; e < 4; ++e) part = fmaf(bf16hi(gw[e]), bf16hi(ow[e]), fmaf(bf16lo(gw[e]), bf16lo(ow[e]), part));
      }
      Dq = sum_with_other_half(part);
    }
  }
  const float2* rope_row = p.rope_table ? reinterpret_cast<const float2*>(p.rope_table) + (size_t)orig_q * (D / 2) : nullptr;
  if (rope_row) {
    // Q arrives unrotated: RoPE on the query's original position (App. B, App. C; Sec. 4.2), as in the forward;
    // the rotated rows are left for the dK/dV kernel
    rope_row_fragments<D>(qf, rope_row, g2, p.rope_interleaved);
    if (s < n) {
      bf16_t* qrow = reinterpret_cast<bf16_t*>(p.Q_rot) + (head_row0 + orig_q) * D;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) *reinterpret_cast<bf16x8*>(qrow + 16 * kk + 8 * g2) = qf[kk];
    }
  }
  const float lse2 = p.lse_in[head_row0 + orig_q] * kLog2e;
  if (p.O_rows) {
    if (g2 == 0 && s < n) p.Dsum_out[head_row0 + orig_q] = Dq;
  } else {
    Dq = p.Dsum[head_row0 + orig_q];
  }

  int koff[D / 16], troff[D / 32][2];
  swizzled_row_offsets<D>(lane, koff);
  swizzled_tr_offsets<D>(lane, troff);

  const int Ll = circular ? L : min(L, max(s, 0));
  const int Rl = circular ? R : min(R, max(n - 1 - s, 0));
  const unsigned LRl = (unsigned)(Ll + Rl);
  const float cs = p.scale * kLog2e;
  const s16x2 oq1 = {(short)(orig_q + 1 - 32768), (short)(orig_q + 1 - 32768)};

  f32x16 dqacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;

  for (int tile = 0; tile < ntiles; ++tile) {
    const int buf = tile & 1;
    // this wave's share of the tile has landed; after the barrier the whole tile is visible and everyone
    // is done with the other buffer (the tile before, the staging of the prologue)
    wait_all_loads();
    __syncthreads();
    if (tile + 1 < ntiles) {
      request_tile(buf ^ 1);
      if (tile + 2 < ntiles) load_idx(tile + 2);
    }
    const bf16_t* Ks = reinterpret_cast<const bf16_t*>(smem + buf * C::BUF_BYTES);
    const bf16_t* Vs = reinterpret_cast<const bf16_t*>(smem + buf * C::BUF_BYTES + C::TILE_BYTES);
    const int* pk_lds = reinterpret_cast<const int*>(smem + C::AREA_BYTES + buf * C::SLOT_BYTES);
    const short* pk16_lds = reinterpret_cast<const short*>(smem + C::AREA_BYTES + buf * C::SLOT_BYTES);
    const int t0 = t_lo + tile * BN;
#pragma unroll
    for (int kb = 0; kb < BN / 32; ++kb) {
      const int tb0 = t0 + 32 * kb;
      const int dmax = tb0 + 31 - s_w0, dmin = tb0 - (s_w0 + 31);
      const bool act = !(dmax < -L || dmin > R) && tb0 <= t_hi;
      const bool inside = dmin >= -L && dmax <= R && tb0 + 31 <= t_hi && s_w0 + 31 <= q_last;
      if (!act) continue;
      f32x16 sacc, dpacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
      {
        // the operand reads of step kk + 1 are under way while the matrix instructions of step kk issue (left
        // to itself the compiler reads every step into the same registers, one LDS latency per step)
        bf16x8 ka[2], va[2];
        ka[0] = *reinterpret_cast<const bf16x8*>(Ks + 32 * kb * D + koff[0]);
        va[0] = *reinterpret_cast<const bf16x8*>(Vs + 32 * kb * D + koff[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
          if (kk + 1 < D / 16) {
            ka[(kk + 1) & 1] = *reinterpret_cast<const bf16x8*>(Ks + 32 * kb * D + koff[kk + 1]);
            va[(kk + 1) & 1] = *reinterpret_cast<const bf16x8*>(Vs + 32 * kb * D + koff[kk + 1]);
            __builtin_amdgcn_sched_barrier(0);
          }
          sacc = mfma_bf16(ka[kk & 1], qf[kk], sacc);    // S^T = K Q^T
          dpacc = mfma_bf16(va[kk & 1], gf[kk], dpacc);  // dP^T = V dO^T
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (CAUSAL == CAUSAL_I32) {
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
      bf16x8 dsf0, dsf1;
      if (CAUSAL == CAUSAL_I16) {
        // pair e = accumulators 2e, 2e+1 = dword e of the lane group's 16 positions
        const uint32_t* pk16 = reinterpret_cast<const uint32_t*>(pk16_lds) + 16 * kb + 8 * g2;
        const u32x4 ia = *reinterpret_cast<const u32x4*>(pk16), ib = *reinterpret_cast<const u32x4*>(pk16 + 4);
        u32x4 w[2];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe0 = __builtin_amdgcn_exp2f(fmaf(sacc[2 * e], cs, -lse2));
          const float pe1 = __builtin_amdgcn_exp2f(fmaf(sacc[2 * e + 1], cs, -lse2));
          const s16x2 pk2 = __builtin_bit_cast(s16x2, e < 4 ? ia[e & 3] : ib[e & 3]);
          const s16x2 later = __builtin_elementwise_sub_sat(pk2, oq1);  // >= 0 for keys after the query
          w[e >> 2][e & 3] = pack_bf16(pe0 * (dpacc[2 * e] - Dq), pe1 * (dpacc[2 * e + 1] - Dq)) &
                             __builtin_bit_cast(uint32_t, later >> (short)15);
        }
        dsf0 = __builtin_bit_cast(bf16x8, w[0]);
        dsf1 = __builtin_bit_cast(bf16x8, w[1]);
      } else {
        float ds[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float pe = __builtin_amdgcn_exp2f(fmaf(sacc[i], cs, -lse2));
          ds[i] = pe * (dpacc[i] - Dq);
        }
        dsf0 = pack_b_operand(ds);
        dsf1 = pack_b_operand(ds + 8);
      }
      {  // dQ^T += K^T dS^T: the half of the block's key rows outermost, so that two products on the same
         // accumulator are D / 32 instructions apart; the operand of product m + 1 is read before product m issues
        constexpr int NPQ = 2 * (D / 32);
        bf16x8 ka[2];
        ka[0] = lds_read_transposed_swz(Ks + (32 * kb) * D, troff[0]);
#pragma unroll
        for (int m = 0; m < NPQ; ++m) {
          if (m + 1 < NPQ) {
            ka[(m + 1) & 1] = lds_read_transposed_swz(Ks + (32 * kb + 16 * ((m + 1) / (D / 32))) * D, troff[(m + 1) % (D / 32)]);
            __builtin_amdgcn_sched_barrier(0);
          }
          dqacc[m % (D / 32)] = mfma_bf16(ka[m & 1], m < D / 32 ? dsf0 : dsf1, dqacc[m % (D / 32)]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  __syncthreads();
  bf16_t* stage = reinterpret_cast<bf16_t*>(smem) + wave * 32 * C::STR;
  store_rows<C, D>(dqacc, p.scale, stage, reinterpret_cast<bf16_t*>(p.dQ) + head_row0 * D, st_src, orig_q, s_w0, n, lane,
                   p.accumulate, rope_row, p.rope_interleaved);
}

// --------------------------------------------------------------------------------------- dK, dV
template <int D, int CAUSAL>
__global__ __launch_bounds__(NT, D == 128 ? DKV128_WAVES : DKV64_WAVES) void bwd_dkv_mfma_bf16_kernel(const Pass p, const int num_kt, const long total_work) {
  using C = Cfg<D, D == 64 ? DKV64_BN : DKV128_BN>;
  constexpr int BN = C::BN;
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

  const long work = xcd_work_index(total_work);
  if (work < 0) return;
  const int kt = (int)(work % num_kt);
  long rest = work / num_kt;
  const int hk = (int)(rest % p.Hkv);
  const int b = (int)(rest / p.Hkv);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g2 = lane >> 5, c32 = lane & 31;
  const int n = p.n, L = p.win.L, R = p.win.R;
  const bool circular = p.win.circular != 0;
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
    for (int i = 0; i < 16; ++i) {
      dkacc[db][i] = 0.f;
      dvacc[db][i] = 0.f;
    }

  const int32_t* perm = nullptr;
  const int hg_begin = p.hq_only >= 0 ? p.hq_only : 0;
  const int hg_end = p.hq_only >= 0 ? p.hq_only + 1 : p.g;
  bf16x8 kf[D / 16], vf[D / 16];
  int orig_k = 0;
  int st_src[C::SP];
  const int pq_pos = acc_order_pos(tid & (BN - 1));
  int koff[D / 16], troff[D / 32][2];
  swizzled_row_offsets<D>(lane, koff);
  swizzled_tr_offsets<D>(lane, troff);
  // The products of one block on the output accumulators, as a list: m = half * NP/2 + r, where half selects
  // the block's query rows 0-15 / 16-31 (operand halves 0 / 1 of P and dS) and r runs over the 32-column
  // blocks of the outputs (dV and dK alternate when both are formed), so that two products on the same
  // accumulator are NP/2 instructions apart.
  constexpr int NP = 4 * (D / 32);
  constexpr int PPS = NP / 8;  // products per slot
  constexpr int PF = 1;  // how many steps ahead the operands of S and dP are read (deeper: no gain)
  // One wave per SIMD has nobody to hide its latencies behind: there the products of a block on the outputs
  // wait for the vector work of the next block (16 more registers; at two waves per SIMD they would spill),
  // and S and dP are pinned to the vector half of the register file.
  constexpr bool DEFER = D == 128 && DKV128_WAVES == 1;
  constexpr bool S_IN_VEC = DEFER;
  static_assert(NP % 8 == 0, "a whole number of products per slot");
  auto product_operand = [&](const int m, const bf16_t* Qb, const bf16_t* Gb) -> bf16x8 {
    const int half = m / (NP / 2), r = m % (NP / 2);
    const int db = r / 2;
    const bool is_dv = (r % 2) == 0;
    return lds_read_transposed_swz((is_dv ? Gb : Qb) + 16 * half * D, troff[db]);
  };
  auto product = [&](const int m, const bf16x8 a, const bf16x8* pf, const bf16x8* dsf) {
    const int half = m / (NP / 2), r = m % (NP / 2);
    const int db = r / 2;
    const bool is_dv = (r % 2) == 0;
    if (is_dv) dvacc[db] = mfma_bf16(a, pf[half], dvacc[db]);
    else dkacc[db] = mfma_bf16(a, dsf[half], dkacc[db]);
  };
  for (int hg = hg_begin; hg < hg_end; ++hg) {
    const int hq = hk * p.g + hg;
    const int32_t* __restrict__ perm_h =
        p.perm ? p.perm + (size_t)perm_slice_index(p.perm_B, p.perm_H, b, hq) * n : nullptr;
    // the stationary K and V rows are (re)loaded when the slot order changes; with one permutation
    // per group that is once
    const bool reload = hg == hg_begin || perm_h != perm;
    perm = perm_h;
    const size_t head_row0 = ((size_t)b * p.Hq + hq) * n;
    const bf16_t* __restrict__ Qh = reinterpret_cast<const bf16_t*>(p.Q) + head_row0 * D;
    const bf16_t* __restrict__ dOh = reinterpret_cast<const bf16_t*>(p.dO) + head_row0 * D;
    const float* __restrict__ lse_h = p.lse_in + head_row0;
    const float* __restrict__ dd_h = p.Dsum + head_row0;

    // streamed tiles: Q | dO rows of BN query slots, fetched through the index tensor by direct
    // global-to-LDS loads one tile ahead (double buffered, one barrier per tile), with the per-slot
    // values (causal position, LSE, -D) of the tile beside them.  Row indices are loaded one tile, the
    // slot's own position two tiles, LSE and D one tile before the tile is requested.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const int ld_row = tid / C::VPR;
    const uint32_t ld_chunk_off = (uint32_t)(((tid % C::VPR) ^ swz<D>(ld_row)) * 16);
    auto row_index = [&](int tile, int v) -> int {
      return slot_to_orig(perm, wrap_slot(min(s_lo + tile * BN + v * C::RPP + ld_row, s_hi), n));
    };
    auto slot_position = [&](int tile) -> int {  // tid < BN
      return slot_to_orig(perm, wrap_slot(min(s_lo + tile * BN + tid, s_hi), n));
    };
    int idx[C::NV];
    int pq_w = 0, pq_n = 0;
    float lse_w = 0.f, dd_w = 0.f;
    // instruction j of the request for a tile: j < NV the Q rows whose indices are in idx[j], j >= NV the dO
    // rows of idx[j - NV]
    auto request_instr = [&](const int j, const int buf) {
      const int v = j % C::NV;
      const uint32_t goff = (uint32_t)idx[v] * (uint32_t)(D * 2) + ld_chunk_off;
      const uint32_t at = buf * C::BUF_BYTES + (v * C::RPP + wave * C::WRPP) * (D * 2) + (j < C::NV ? 0 : C::TILE_BYTES);
      load_to_lds_16(j < C::NV ? Qh : dOh, goff, lds0 + at);
    };
    // publishes the per-slot values held in *_w beside the tile that is being requested
    auto publish_slots = [&](const int buf) {
      if (tid < BN) {
        char* slot = smem + C::AREA_BYTES + buf * C::SLOT_BYTES;
        if (CAUSAL == CAUSAL_I32) reinterpret_cast<int*>(slot)[tid] = pq_w;
        if (CAUSAL == CAUSAL_I16) reinterpret_cast<short*>(slot)[pq_pos] = (short)(pq_w - 32767);
        reinterpret_cast<float*>(slot + BN * 4)[tid] = lse_w * kLog2e;
        reinterpret_cast<float*>(slot + 2 * BN * 4)[tid] = -dd_w;  // dP starts from -D, so that the product leaves dP - D
      }
    };
    auto request_tile = [&](const int buf) {
#pragma unroll
      for (int j = 0; j < 2 * C::NV; ++j) request_instr(j, buf);
      publish_slots(buf);
    };
    auto load_slot_values = [&]() {  // LSE and D of the slot whose position is in pq_w
      if (tid < BN) {
        lse_w = lse_h[pq_w];  // used (scaled) when the tile is published: no wait for it among the requests
        dd_w = dd_h[pq_w];
      }
    };
    if (hg != hg_begin) __syncthreads();  // a slower wave may still read the previous head's last tile
    // every index first, then every row (stationary K and V, first Q/dO tile), then the staging
    if (reload) {
      stationary_src<C>(perm, t_w0, n, lane, st_src);
      orig_k = slot_to_orig(perm, min(t, n - 1));
    }
#pragma unroll
    for (int v = 0; v < C::NV; ++v) idx[v] = row_index(0, v);
    int pq_1 = 0;
    if (tid < BN) {
      pq_w = slot_position(0);
      pq_1 = slot_position(1);
      pq_n = slot_position(2);
    }
    load_slot_values();
    if (reload) {
      u32x4 krow[C::SP], vrow[C::SP];
      stationary_rows<C, D>(Kh, st_src, lane, krow);
      stationary_rows<C, D>(Vh, st_src, lane, vrow);
      request_tile(0);
      bf16_t* stage_kv = reinterpret_cast<bf16_t*>(smem + C::BUF_BYTES) + wave * 32 * C::STR;  // buffer 1 is still free
      stationary_put<C>(stage_kv, lane, krow);
      wave_lds_sync();
      stationary_get<C, D>(stage_kv, lane, kf);
      wave_lds_sync();
      stationary_put<C>(stage_kv, lane, vrow);
      wave_lds_sync();
      stationary_get<C, D>(stage_kv, lane, vf);
    } else {
      request_tile(0);
    }
    pq_w = pq_1;
    load_slot_values();
#pragma unroll
    for (int v = 0; v < C::NV; ++v) idx[v] = row_index(1, v);
    // visible iff the query's original position >= the key's: (orig_k - 1) - pq < 0, on positions biased by 32767
    const s16x2 okm1 = {(short)(orig_k - 32768), (short)(orig_k - 32768)};

    for (int tile = 0; tile < ntiles; ++tile) {
      const int buf = tile & 1;
      // this wave's share of the tile has landed; after the barrier the whole tile is visible and
      // everyone is done with the other buffer (the tile before, the staging of the prologue)
      wait_all_loads();
      __syncthreads();
      // the next tile (a direct-to-LDS load holds the wave's issue port for about 100 cycles here, wherever in
      // the tile it is placed and also when the rows travel through registers instead)
      const bool more = tile + 1 < ntiles;
      if (more) {
#pragma unroll
        for (int j = 0; j < 2 * C::NV; ++j) request_instr(j, buf ^ 1);
        publish_slots(buf ^ 1);
        pq_w = pq_n;
        load_slot_values();
#pragma unroll
        for (int v = 0; v < C::NV; ++v) idx[v] = row_index(tile + 2, v);
        if (tid < BN) pq_n = slot_position(tile + 3);
      }
      const bf16_t* Qs = reinterpret_cast<const bf16_t*>(smem + buf * C::BUF_BYTES);
      const bf16_t* Gs = reinterpret_cast<const bf16_t*>(smem + buf * C::BUF_BYTES + C::TILE_BYTES);
      const char* slot = smem + C::AREA_BYTES + buf * C::SLOT_BYTES;
      const int* pq_lds = reinterpret_cast<const int*>(slot);
      const short* pq16_lds = reinterpret_cast<const short*>(slot);
      const float* lse_lds = reinterpret_cast<const float*>(slot + BN * 4);
      const float* dd_lds = reinterpret_cast<const float*>(slot + 2 * BN * 4);
      const int s0 = s_lo + tile * BN;
      bool pend = false;
      bf16x8 pfP[2], dsfP[2];
      const bf16_t *QsP = Qs, *GsP = Gs;
#pragma unroll
      for (int qb = 0; qb < BN / 32; ++qb) {
        const int sb0 = s0 + 32 * qb;
        const int dmax = t_w0 + 31 - sb0, dmin = t_w0 - (sb0 + 31);  // range of t - s over the block
        const bool act = !(dmax < -L || dmin > R) && sb0 <= s_hi;
        const bool inside = dmin >= -L && dmax <= R && sb0 + 31 <= s_hi && t_w0 + 31 <= t_last;
        if (!act) continue;
        f32x16 sacc, dpacc;
#pragma unroll
        for (int mq = 0; mq < 4; ++mq) {
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(dd_lds + 32 * qb + 8 * mq + 4 * g2);
#pragma unroll
          for (int x = 0; x < 4; ++x) { sacc[4 * mq + x] = 0.f; dpacc[4 * mq + x] = d4[x]; }
        }
        {
          // the operand reads of steps kk + 1 .. kk + PF are under way while the matrix instructions of step kk issue
          // (left to itself the compiler reads every step into the same registers, one LDS latency per step)
          constexpr int NB = PF + 1;
          bf16x8 qa[NB], ga[NB];
#pragma unroll
          for (int j = 0; j < PF; ++j) {
            qa[j] = *reinterpret_cast<const bf16x8*>(Qs + 32 * qb * D + koff[j]);
            ga[j] = *reinterpret_cast<const bf16x8*>(Gs + 32 * qb * D + koff[j]);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int kk = 0; kk < D / 16; ++kk) {
            if (kk + PF < D / 16) {
              qa[(kk + PF) % NB] = *reinterpret_cast<const bf16x8*>(Qs + 32 * qb * D + koff[kk + PF]);
              ga[(kk + PF) % NB] = *reinterpret_cast<const bf16x8*>(Gs + 32 * qb * D + koff[kk + PF]);
              __builtin_amdgcn_sched_barrier(0);
            }
            if (S_IN_VEC) {
              if (kk == 0) mfma_bf16_v_first(qa[0], kf[0], sacc);
              else mfma_bf16_v(qa[kk % NB], kf[kk], sacc);
              mfma_bf16_v(ga[kk % NB], vf[kk], dpacc);
            } else {
              sacc = mfma_bf16(qa[kk % NB], kf[kk], sacc);    // S = Q K^T
              dpacc = mfma_bf16(ga[kk % NB], vf[kk], dpacc);  // dP = dO V^T
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          if (S_IN_VEC) matrix_results_to_vector(sacc, dpacc);
        }
        // accumulator i is query row 32*qb + 8*(i/4) + 4*g2 + i%4 of the tile, key column = lane
        if (CAUSAL == CAUSAL_I32) {
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
        // P and dS of this block, pair by pair (accumulators 2e, 2e+1), while the matrix pipe works off the
        // products of the block before it (dV^T += dO^T P, dK^T += Q^T dS: contraction over its 32 query rows),
        // whose operands wait in pfP / dsfP: one slot per pair = its share of the matrix instructions, the
        // operand reads of the next slot, the pair's vector work; nothing moves across a slot boundary.
        f32x4 l4[4];
#pragma unroll
        for (int mq = 0; mq < 4; ++mq) l4[mq] = *reinterpret_cast<const f32x4*>(lse_lds + 32 * qb + 8 * mq + 4 * g2);
        u32x4 ia = {0, 0, 0, 0}, ib = {0, 0, 0, 0};
        if (CAUSAL == CAUSAL_I16) {
          const uint32_t* pq16 = reinterpret_cast<const uint32_t*>(pq16_lds) + 16 * qb + 8 * g2;
          ia = *reinterpret_cast<const u32x4*>(pq16);
          ib = *reinterpret_cast<const u32x4*>(pq16 + 4);
        }
        u32x4 wp[2], wd[2];
        auto pair = [&](const int e) {
          const int i0 = 2 * e, i1 = 2 * e + 1;
          const float pe0 = __builtin_amdgcn_exp2f(fmaf(sacc[i0], cs, -l4[i0 >> 2][i0 & 3]));
          const float pe1 = __builtin_amdgcn_exp2f(fmaf(sacc[i1], cs, -l4[i1 >> 2][i1 & 3]));
          uint32_t vis = 0xffffffffu;
          if (CAUSAL == CAUSAL_I16) {
            const s16x2 pq2 = __builtin_bit_cast(s16x2, e < 4 ? ia[e & 3] : ib[e & 3]);
            vis = __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(okm1, pq2) >> (short)15);
          }
          wp[e >> 2][e & 3] = pack_bf16(pe0, pe1) & vis;
          wd[e >> 2][e & 3] = pack_bf16(pe0 * dpacc[i0], pe1 * dpacc[i1]) & vis;  // dpacc = dP - D
        };
        if (pend) {
          bf16x8 aop[2][PPS];
#pragma unroll
          for (int j = 0; j < PPS; ++j) aop[0][j] = product_operand(j, QsP, GsP);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (e + 1 < 8) {
#pragma unroll
              for (int j = 0; j < PPS; ++j) aop[(e + 1) & 1][j] = product_operand((e + 1) * PPS + j, QsP, GsP);
            }
#pragma unroll
            for (int j = 0; j < PPS; ++j) product(e * PPS + j, aop[e & 1][j], pfP, dsfP);
            pair(e);
            __builtin_amdgcn_sched_barrier(0);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) pair(e);
        }
        pfP[0] = __builtin_bit_cast(bf16x8, wp[0]); pfP[1] = __builtin_bit_cast(bf16x8, wp[1]);
        dsfP[0] = __builtin_bit_cast(bf16x8, wd[0]); dsfP[1] = __builtin_bit_cast(bf16x8, wd[1]);
        QsP = Qs + 32 * qb * D;
        GsP = Gs + 32 * qb * D;
        if (DEFER) {
          pend = true;
        } else {
#pragma unroll
          for (int m = 0; m < NP; ++m) product(m, product_operand(m, QsP, GsP), pfP, dsfP);
        }
      }
      if (pend) {  // the last block of the tile: its rows are overwritten after the next barrier
#pragma unroll
        for (int m = 0; m < NP; ++m) product(m, product_operand(m, QsP, GsP), pfP, dsfP);
      }
    }
  }
  __syncthreads();
  bf16_t* dKh = reinterpret_cast<bf16_t*>(p.dK) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  bf16_t* dVh = reinterpret_cast<bf16_t*>(p.dV) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  const float2* rope_row = p.rope_dk ? reinterpret_cast<const float2*>(p.rope_table) + (size_t)orig_k * (D / 2) : nullptr;
  store_rows<C, D>(dkacc, p.scale, stage, dKh, st_src, orig_k, t_w0, n, lane, p.accumulate, rope_row, p.rope_interleaved);
  store_rows<C, D>(dvacc, 1.f, stage, dVh, st_src, orig_k, t_w0, n, lane, p.accumulate);
}

inline int causal_mode(const Pass& p) {
  // identity order with a one-sided linear window (plain causal SWA): the window already excludes every
  // later key, the causal test would only repeat it
  const bool window_is_causal = !p.perm && !p.win.circular && p.win.R == 0;
  return (!p.causal || window_is_causal) ? CAUSAL_NONE : (p.n <= 65535 ? CAUSAL_I16 : CAUSAL_I32);
}

template <int D>
hipError_t launch_dq_t(const Pass& p, hipStream_t st) {
  // Query heads of a KV group that read K/V through the same permutation (or none) share a workgroup
  const bool shared_perm = !p.perm || p.perm_H == 1;
  const int hshift = !shared_perm ? 0 : (p.g % 4 == 0 ? 2 : (p.g % 2 == 0 ? 1 : 0));
  const int bm = BM >> hshift;
  const int num_qt = (p.n + bm - 1) / bm;
  const long total = (long)num_qt * (p.Hq >> hshift) * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(NT);
  switch (causal_mode(p)) {
    case CAUSAL_NONE: hipLaunchKernelGGL((bwd_dq_mfma_bf16_kernel<D, CAUSAL_NONE>), grid, block, 0, st, p, num_qt, total, hshift); break;
    case CAUSAL_I16: hipLaunchKernelGGL((bwd_dq_mfma_bf16_kernel<D, CAUSAL_I16>), grid, block, 0, st, p, num_qt, total, hshift); break;
    default: hipLaunchKernelGGL((bwd_dq_mfma_bf16_kernel<D, CAUSAL_I32>), grid, block, 0, st, p, num_qt, total, hshift); break;
  }
  return hipGetLastError();
}

template <int D>
hipError_t launch_dkv_t(const Pass& p, hipStream_t st) {
  const int num_kt = (p.n + BM - 1) / BM;
  const long total = (long)num_kt * p.Hkv * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(NT);
  switch (causal_mode(p)) {
    case CAUSAL_NONE: hipLaunchKernelGGL((bwd_dkv_mfma_bf16_kernel<D, CAUSAL_NONE>), grid, block, 0, st, p, num_kt, total); break;
    case CAUSAL_I16: hipLaunchKernelGGL((bwd_dkv_mfma_bf16_kernel<D, CAUSAL_I16>), grid, block, 0, st, p, num_kt, total); break;
    default: hipLaunchKernelGGL((bwd_dkv_mfma_bf16_kernel<D, CAUSAL_I32>), grid, block, 0, st, p, num_kt, total); break;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_mfma_bf16(const Pass& p, hipStream_t st) {
  if (p.n < 1 || p.B < 1 || p.Hq < 1 || p.Hkv < 1 || p.g * p.Hkv != p.Hq) return hipErrorInvalidValue;
  if (p.win.L < 0 || p.win.R < 0 || p.win.L >= p.n || p.win.R >= p.n) return hipErrorInvalidValue;
  if (p.win.circular && p.win.L + p.win.R + 1 > p.n) return hipErrorInvalidValue;
  if (!p.dO || !p.lse_in || !p.dQ || !p.dK || !p.dV) return hipErrorInvalidValue;
  if (p.O_rows ? !p.Dsum_out : !p.Dsum) return hipErrorInvalidValue;
  if (!(p.d == 64 || p.d == 128)) return hipErrorNotSupported;
  if ((long)p.n * p.d * 2 >= (1L << 31)) return hipErrorNotSupported;  // 32-bit row offsets inside a head
  if (p.rope_dk && !p.rope_table) return hipErrorInvalidValue;
  if (p.rope_table && !p.Q_rot) return hipErrorInvalidValue;
  hipError_t e = p.d == 64 ? launch_dq_t<64>(p, st) : launch_dq_t<128>(p, st);
  if (e != hipSuccess) return e;
  Pass kv = p;
  if (p.rope_table) kv.Q = p.Q_rot;  // the dQ kernel has left the rotated rows there
  if (p.O_rows) kv.Dsum = p.Dsum_out;  // and the row sums here
  if (p.perm && p.perm_H != 1 && p.g > 1) {
    // every query head of a group has its own slot order: one pass per head, summed in place
    Pass q = kv;
    for (int hg = 0; hg < p.g; ++hg) {
      q.hq_only = hg;
      q.accumulate = (hg == 0) ? p.accumulate : 1;
      e = p.d == 64 ? launch_dkv_t<64>(q, st) : launch_dkv_t<128>(q, st);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  return p.d == 64 ? launch_dkv_t<64>(kv, st) : launch_dkv_t<128>(kv, st);
}

}  // namespace sa
