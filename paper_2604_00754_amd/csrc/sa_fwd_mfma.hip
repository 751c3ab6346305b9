// bf16 forward of Stochastic Attention on gfx950 matrix cores.
//
// One workgroup (4 wavefronts) owns 128 query rows of one (batch, KV head); a wavefront owns 32
// consecutive PERMUTED slots of one query head.  Without grouped heads the four wavefronts take four
// adjacent 32-slot blocks of the same query head.  When the query heads of a KV group share one
// permutation (App. B: one permutation per layer), the wavefronts instead take the SAME slots of up
// to four query heads of the group: all of them then need exactly the same K/V rows, so the band the
// workgroup walks is 32 + w slots instead of 128 + w and no wavefront idles on tiles outside its own
// band.  The workgroup walks the slots of the window band (Eq. 3) in tiles of
// 64; K and V rows of a tile are read through the index tensor straight from their original
// positions (the permuted copies of Alg. 1 never exist) by direct global-to-LDS loads, one tile ahead
// (no registers, no LDS stores; rows unpadded, 16-byte chunks XOR-swizzled; double buffered, one
// barrier per tile), and consumed by
//   S^T = K Q^T          (v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q held in registers)
//   mask: window on slot offsets, causal test on original positions (Sec. 3.3, App. B)
//   softmax (Eq. 1) -- in the S^T layout a lane holds one query column, so row statistics are lane-local
//   up to one exchange with lane^32.  A workgroup first walks its band with the softmax reference fixed
//   at zero (p = exp2(cs * s): no maximum, no rescaling; O and l carry the same reference, so O / l does
//   not depend on it) and looks at the row sums at the end; only if one of them left the range that form
//   holds in fp32 does it walk the band again in the online form, with a running maximum that is moved
//   when a tile exceeds it by more than 2^8
//   O^T += V^T P^T       (A = V^T gathered from the row-major V tile by transposing LDS reads,
//                         ds_read_b64_tr_b16; B = P^T taken directly from the S^T accumulators)
// The epilogue normalises, transposes through LDS and writes each row to its ORIGINAL position
// (the "undo permute" of Alg. 1), optionally forming the gated sum of Eq. 5 on the way out.
#include <type_traits>

#include "sa_common.h"
#include "sa_mfma.h"

namespace sa {
namespace {

#ifndef FWD_BN64
#define FWD_BN64 64
#endif
#ifndef FWD_WGS64
#define FWD_WGS64 4
#endif
#ifndef FWD_BN128
#define FWD_BN128 32
#endif
#ifndef FWD_KG128
#define FWD_KG128 4
#endif
#ifndef FWD_WGS128
#define FWD_WGS128 3
#endif
constexpr int BM = 128;  // query rows per workgroup (slots x heads)
constexpr int NT = 256;  // threads per workgroup

template <int D>
struct Cfg {
  static constexpr int BN = D == 128 ? FWD_BN128 : FWD_BN64;  // key slots per tile
  static constexpr int NB = BN / 32;     // 32-slot blocks per tile
  static constexpr int QSTR = D + 8;     // bf16 per row of the Q / O staging area: +16 B keeps 16 consecutive rows on distinct banks for 16-byte reads
  static constexpr int CPR = D / 8;      // 16-byte chunks per K/V row
  static constexpr int RPI = 64 / CPR;   // K/V rows one wave moves with one 16-byte-per-lane instruction
  static constexpr int NI = BN / (4 * RPI);  // such instructions per wave, tile and operand
  static constexpr int WRPP = 64 / CPR;  // rows covered by one pass of a single wave
  static constexpr int TILE_BYTES = BN * D * 2;      // one operand tile, rows unpadded
  static constexpr int BUF_BYTES = 2 * TILE_BYTES;   // K | V
  static constexpr int QBYTES = 4 * 32 * QSTR * 2;   // per-wave Q / O staging; starts at a buffer and runs past its end
  static constexpr int RING = 4;                     // tiles whose row indices are kept in LDS
  static constexpr int RING_OFF = BUF_BYTES + QBYTES;  // buffer 0 | buffer 1 = start of the staging area | its overhang
  static constexpr int LDS_BYTES = RING_OFF + RING * BN * 6 + BM * 4;  // ... | index ring | 16-bit index ring | row stash
  static_assert(QBYTES >= BUF_BYTES, "the staging area covers buffer 1");
  static_assert(BUF_BYTES % 16 == 0 && QBYTES % 16 == 0, "everything stays 16-byte aligned");
};

// 16-byte chunk `chunk` of row `row` of a [n, D] bf16 head: a 32-bit byte offset from the (wave-uniform)
// head pointer, so the address needs one vector instruction (the host checks n * D * 2 < 2^31).
template <int D>
__device__ __forceinline__ u32x4 load_row_chunk(const bf16_t* head, int row, int chunk) {
  const uint32_t off = (uint32_t)row * (uint32_t)(D * 2) + (uint32_t)chunk * 16u;
  return *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(head) + off);
}

// The same for rows that are read once (the query rows): a non-temporal load, so that the streamed rows do
// not displace the K/V rows that neighbouring workgroups share in L2.
template <int D>
__device__ __forceinline__ u32x4 load_row_chunk_once(const bf16_t* head, int row, int chunk) {
  const uint32_t off = (uint32_t)row * (uint32_t)(D * 2) + (uint32_t)chunk * 16u;
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(head) + off));
}

// Causal test modes.  CAUSAL_NONE: no test.  CAUSAL_I32: scores of later keys are set to -inf before
// the softmax (any n).  CAUSAL_I16 (n <= 65535): the probabilities of later keys are cleared after
// they are packed to bf16 pairs, with packed 16-bit compares on biased original indices.
enum { CAUSAL_NONE = 0, CAUSAL_I32 = 1, CAUSAL_I16 = 2 };

// PERM = false: identity permutation (plain windowed attention); no index loads are generated.
// GATED = true: the second branch of the gated forward, with the gated sum of Eq. 5 in the epilogue; it needs
// more registers after the tile loop, so at d = 64 it runs three workgroups per CU where the plain kernel
// runs four.
template <int D, bool PERM, int CAUSAL, bool GATED>
__global__ __launch_bounds__(NT, D == 64 ? (GATED ? 3 : FWD_WGS64) : (GATED ? 2 : FWD_WGS128)) void fwd_mfma_bf16_kernel(const Pass p, const int num_qt, const long total_work,
                                                              const int hshift) {
  using C = Cfg<D>;
  constexpr int BN = C::BN, NB = C::NB;
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

  // 1 << hshift = query heads per workgroup (1, 2 or 4; a divisor of the group size).  Work list order: the
  // head sets of a KV group, then the next query tile -- neighbours share K/V rows
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
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
  const int hq = hk * p.g + (hset << hshift) + (wave & ((1 << hshift) - 1));  // this wave's query head
  const int bm = BM >> hshift;                                               // query slots of the workgroup
  const int g2 = lane >> 5, c32 = lane & 31;
  const int n = p.n, L = p.win.L, R = p.win.R;
  const bool circular = p.win.circular != 0;
  const int32_t* __restrict__ perm =
      PERM ? p.perm + (size_t)perm_slice_index(p.perm_B, p.perm_H, b, hq) * n : nullptr;
  auto orig_of = [&](int slot) -> int { return PERM ? perm[slot] : slot; };
  const bf16_t* __restrict__ Qh = reinterpret_cast<const bf16_t*>(p.Q) + ((size_t)b * p.Hq + hq) * n * (size_t)D;
  const bf16_t* __restrict__ Kh = reinterpret_cast<const bf16_t*>(p.K) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;
  const bf16_t* __restrict__ Vh = reinterpret_cast<const bf16_t*>(p.V) + ((size_t)b * p.Hkv + hk) * n * (size_t)D;

  const int p0 = qt * bm;
  const int q_last = min(p0 + bm - 1, n - 1);
  const int s_w0 = p0 + 32 * (wave >> hshift);  // first query slot of this wave
  const int s = s_w0 + c32;         // this lane's query slot (column of S^T)
  const int orig_q = orig_of(min(s, n - 1));

  // key-slot range of the workgroup, unwrapped
  int t_lo = p0 - L, t_hi = q_last + R;
  if (!circular) {
    t_lo = max(t_lo, 0);
    t_hi = min(t_hi, n - 1);
  }
  const int ntiles = (t_hi - t_lo + BN) / BN;

  // ---- original indices of the rows of tiles 0..2 go to the LDS ring; tile 3's stay in a register
  int* ring = reinterpret_cast<int*>(smem + C::RING_OFF);
  auto tile_row_orig = [&](int tile) -> int {  // original index of row `tid` of a tile (clamped to the range)
    return orig_of(wrap_slot(min(t_lo + tile * BN + tid, t_hi), n));
  };
  // CAUSAL_I16 keeps a second copy for the mask: index - 32768 as int16, ordered so that a lane's 16
  // accumulators of a block (key rows 8*(i/4) + 4*g2 + i%4) are 32 contiguous bytes
  short* ring16 = reinterpret_cast<short*>(smem + C::RING_OFF + C::RING * BN * 4);
  const int pos16 = (tid & 32) | ((tid & 4) << 2) | ((tid >> 1) & 12) | (tid & 3);  // row tid -> (kb, g2, i)
  // ---- prologue.  All index loads first (this lane's query, the wave's query rows, the rows of tiles
  // 0..3); then, one memory round trip later, the Q rows and the K/V rows of tile 0 together.
  constexpr int NP = 32 / C::WRPP;
  const int chunk16 = lane % C::CPR;
  int src[NP];
#pragma unroll
  for (int pass = 0; pass < NP; ++pass) src[pass] = orig_of(min(s_w0 + pass * C::WRPP + lane / C::CPR, n - 1));
  int* rowstash = reinterpret_cast<int*>(smem + C::RING_OFF + C::RING * BN * 6);  // original index of the workgroup's 128 rows
  int pk_reg = 0;
  auto init_ring = [&]() {  // indices of tiles 0..2 -> ring, tile 3 -> register (the state the tile loop starts from)
    if (tid < BN) {
      const int i0 = tile_row_orig(0), i1 = tile_row_orig(1), i2 = tile_row_orig(2);
      pk_reg = tile_row_orig(3);
      ring[0 * BN + tid] = i0;
      ring[1 * BN + tid] = i1;
      ring[2 * BN + tid] = i2;
      if (CAUSAL == CAUSAL_I16) {
        ring16[0 * BN + pos16] = (short)(i0 - 32768);
        ring16[1 * BN + pos16] = (short)(i1 - 32768);
        ring16[2 * BN + pos16] = (short)(i2 - 32768);
      }
    }
  };
  init_ring();
  if (chunk16 == 0) {
#pragma unroll
    for (int pass = 0; pass < NP; ++pass) rowstash[wave * 32 + pass * C::WRPP + lane / C::CPR] = src[pass];
  }
  __syncthreads();  // ring visible

  // ---- tile loader: direct global-to-LDS loads, 16 bytes per lane.  One instruction of a wave fills RPI
  // consecutive rows of the tile; lane l delivers physical chunk l % CPR of row l / CPR, i.e. fetches the
  // logical chunk (l % CPR) ^ swz(row) of the row the index ring names.  The swizzle depends on the low
  // four bits of the row only, which are the same for every instruction of the lane.
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const int ld_row = wave * C::RPI + lane / C::CPR;  // row of the lane in instruction 0
  const uint32_t ld_chunk_off = (uint32_t)(((lane % C::CPR) ^ swz<D>(ld_row)) * 16);
  auto load_tile = [&](const int tile, const int buf) {
    const int* idx = ring + (tile & (C::RING - 1)) * BN;
    int ridx[C::NI];
#pragma unroll
    for (int j = 0; j < C::NI; ++j) ridx[j] = idx[j * 4 * C::RPI + ld_row];
#pragma unroll
    for (int j = 0; j < C::NI; ++j) {
      const uint32_t goff = (uint32_t)ridx[j] * (uint32_t)(D * 2) + ld_chunk_off;
      const uint32_t dst = lds0 + buf * C::BUF_BYTES + (j * 4 * C::RPI + wave * C::RPI) * (D * 2);
      load_to_lds_16(Kh, goff, dst);
      load_to_lds_16(Vh, goff, dst + C::TILE_BYTES);
    }
  };

  // ---- this wave's 32 query rows go through LDS (second buffer) and are kept as B operands
  bf16_t* Qs = reinterpret_cast<bf16_t*>(smem + C::BUF_BYTES) + wave * 32 * C::QSTR;
  {
    u32x4 v[NP];
#pragma unroll
    for (int pass = 0; pass < NP; ++pass) v[pass] = load_row_chunk_once<D>(Qh, src[pass], chunk16);
    load_tile(0, 0);  // buffer 0 is not the Q staging area
#pragma unroll
    for (int pass = 0; pass < NP; ++pass)
      *reinterpret_cast<u32x4*>(Qs + (pass * C::WRPP + lane / C::CPR) * C::QSTR + chunk16 * 8) = v[pass];
  }
  wave_lds_sync();  // Q rows staged: the rows are this wave's own (tile 0 is waited for at the top of the tile loop,
                    // whose barrier also tells everyone that the staging area may take tile 1)
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8*>(Qs + c32 * C::QSTR + 16 * kk + 8 * g2);
  // RoPE on the query's ORIGINAL position (App. B, App. C; Sec. 4.2), applied to the operand fragments
  if (p.rope_table)
    rope_row_fragments<D>(qf, reinterpret_cast<const float2*>(p.rope_table) + (size_t)orig_q * (D / 2), g2, p.rope_interleaved);

  // ---- per-lane element offsets of the operand reads inside a swizzled tile (without the block's rows)
  int koff[D / 16], voff[D / 32][2];
  swizzled_row_offsets<D>(lane, koff);
  swizzled_tr_offsets<D>(lane, voff);

  const float cs = p.scale * kLog2e;  // exp(scale*x) = exp2(cs*x)
  const float lazy = 8.0f / cs;       // move the reference maximum only for jumps above 2^8
  float m_ref = -INFINITY, l_run = 0.f;
  f32x16 oacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;

  // one tile; BUF (0/1) is a compile-time constant so that all LDS addresses are immediates
  auto do_tile = [&](const int tile, auto bufc, auto fastc) {
    constexpr int buf = decltype(bufc)::value;
    constexpr bool FAST = decltype(fastc)::value;
    // this wave's share of the tile has landed; after the barrier the whole tile is visible and everyone
    // is done with the other buffer (tile-1, Q staging)
    wait_all_loads();
    __syncthreads();
    if (tid < BN) {  // indices: tile+3 -> ring, tile+4 -> register
      ring[((tile + 3) & (C::RING - 1)) * BN + tid] = pk_reg;
      if (CAUSAL == CAUSAL_I16) {
        int te = tid;  // the position is formed again from a copy the optimiser cannot hoist, not kept in a register
        asm volatile("" : "+v"(te));
        const int pos = (te & 32) | ((te & 4) << 2) | ((te >> 1) & 12) | (te & 3);
        ring16[((tile + 3) & (C::RING - 1)) * BN + pos] = (short)(pk_reg - 32768);
      }
      if (tile + 4 < ntiles) pk_reg = tile_row_orig(tile + 4);
    }
    if (tile + 1 < ntiles) load_tile(tile + 1, buf ^ 1);
    const bf16_t* Ks = reinterpret_cast<const bf16_t*>(smem + buf * C::BUF_BYTES);
    const bf16_t* Vs = reinterpret_cast<const bf16_t*>(smem + buf * C::BUF_BYTES + C::TILE_BYTES);
    const int* pk_lds = ring + (tile & (C::RING - 1)) * BN;

    const int t0 = t_lo + tile * BN;
    bool act[NB], inside[NB];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
      const int tb0 = t0 + 32 * kb;
      const int dmax = tb0 + 31 - s_w0, dmin = tb0 - (s_w0 + 31);
      act[kb] = !(dmax < -L || dmin > R) && tb0 <= t_hi;
      inside[kb] = dmin >= -L && dmax <= R && tb0 + 31 <= t_hi && s_w0 + 31 <= q_last;
    }
    bool any_act = false;
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) any_act = any_act || act[kb];
    if (!any_act) return;

    // ---- S^T = K Q^T for the active 32-slot blocks
    f32x16 sacc[NB];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
      if (act[kb]) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
        // the K operands of the block are requested KG at a time, each group before its first product
        constexpr int KG = D == 128 ? FWD_KG128 : D / 16;
#pragma unroll
        for (int k0 = 0; k0 < D / 16; k0 += KG) {
          bf16x8 ka[KG];
#pragma unroll
          for (int kk = 0; kk < KG; ++kk) ka[kk] = *reinterpret_cast<const bf16x8*>(Ks + 32 * kb * D + koff[k0 + kk]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int kk = 0; kk < KG; ++kk) sacc[kb] = mfma_bf16(ka[kk], qf[k0 + kk], sacc[kb]);
          if (k0 + KG < D / 16) __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kb][i] = -INFINITY;
      }
    }

    auto causal_to_neg_inf = [&](f32x16& a, int kb) {
#pragma unroll
      for (int mq = 0; mq < 4; ++mq) {
        const int4 pk = *reinterpret_cast<const int4*>(pk_lds + 32 * kb + 8 * mq + 4 * g2);
        if (pk.x > orig_q) a[4 * mq + 0] = -INFINITY;
        if (pk.y > orig_q) a[4 * mq + 1] = -INFINITY;
        if (pk.z > orig_q) a[4 * mq + 2] = -INFINITY;
        if (pk.w > orig_q) a[4 * mq + 3] = -INFINITY;
      }
    };
    // ---- mask.  Accumulator i of block kb is key row 32*kb + 8*(i/4) + 4*g2 + i%4 of the tile.
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
      if (!act[kb]) continue;
      if (CAUSAL == CAUSAL_I32) causal_to_neg_inf(sacc[kb], kb);
      if (!inside[kb]) {
        // per-lane window constants: key t is visible iff 0 <= t - s + Ll <= LRl (unsigned compare).  Formed
        // here, in the few blocks at the edge of the band, from a copy of s the optimiser cannot hoist.
        int se = lane;
        asm volatile("" : "+v"(se));
        se = s_w0 + (se & 31);
        const int Ll = circular ? L : min(L, max(se, 0));
        const int Rl = circular ? R : min(R, max(n - 1 - se, 0));
        const unsigned LRl = (unsigned)(Ll + Rl);
        const int base = t0 + 32 * kb + 4 * g2 - se + Ll;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const unsigned u = (unsigned)(base + 8 * (i / 4) + (i % 4));
          if (u > LRl) sacc[kb][i] = -INFINITY;
        }
      }
    }

    // ---- softmax (Eq. 1) on the lane's query column.  FAST: reference zero, nothing to do before the
    // exponentials.  Otherwise the online form with a lazily updated reference maximum:
    // p = exp2(cs*(s - m_ref)) stays <= 2^8, and O and l carry the same reference, so O/l is unchanged
    if (!FAST) {
    float mx = sacc[0][0];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][i]);
    mx = max_with_other_half(mx);
    if (__any(mx > m_ref + lazy)) {  // (-inf + lazy = -inf: the first visible key always triggers)
      if (CAUSAL == CAUSAL_I16) {
        // mx still counts later keys (their probabilities are cleared further down, whatever they
        // are): take the maximum over the visible keys only before moving the reference
        float mv = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < NB; ++kb) {
          if (!act[kb]) continue;
          f32x16 t = sacc[kb];
          causal_to_neg_inf(t, kb);
#pragma unroll
          for (int i = 0; i < 16; ++i) mv = fmaxf(mv, t[i]);
        }
        mx = max_with_other_half(mv);
      }
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = (mx > m_ref + lazy) ? __builtin_amdgcn_exp2f((m_ref - m_new) * cs) : 1.f;
      if (mx > m_ref + lazy) m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
    }
    }
    const float mc = FAST ? 0.f : (m_ref == -INFINITY ? 0.f : m_ref) * cs;
    bf16x8 pf[NB][2];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
      if (!act[kb]) continue;
      if (CAUSAL == CAUSAL_I16) {
        // pair e of the lane = accumulators 2e, 2e+1; the ring keeps their biased indices as one dword
        typedef short s16x2 __attribute__((ext_vector_type(2)));
        int oqe = orig_q;  // a copy the optimiser cannot hoist: the packed constant is formed per block, not kept
        asm volatile("" : "+v"(oqe));
        const s16x2 oq1 = {(short)(oqe + 1 - 32768), (short)(oqe + 1 - 32768)};
        const bf16x2 ones = {(bf16_t)1.f, (bf16_t)1.f};
        int ge = lane;
        asm volatile("" : "+v"(ge));
        const uint32_t* pk16 = reinterpret_cast<const uint32_t*>(ring16 + (tile & (C::RING - 1)) * BN) + 16 * kb + 8 * (ge >> 5);
        const u32x4 ia = *reinterpret_cast<const u32x4*>(pk16), ib = *reinterpret_cast<const u32x4*>(pk16 + 4);
        u32x4 w[2];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][2 * e], cs, -mc));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][2 * e + 1], cs, -mc));
          const s16x2 pk2 = __builtin_bit_cast(s16x2, e < 4 ? ia[e & 3] : ib[e & 3]);
          const s16x2 later = __builtin_elementwise_sub_sat(pk2, oq1);  // >= 0 for keys after the query
          const uint32_t pp = pack_bf16(p0, p1) & __builtin_bit_cast(uint32_t, later >> (short)15);
          l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pp), ones, l_run, false);
          w[e >> 2][e & 3] = pp;
        }
        pf[kb][0] = __builtin_bit_cast(bf16x8, w[0]);
        pf[kb][1] = __builtin_bit_cast(bf16x8, w[1]);
      } else {
        // the row sum is taken from the bf16 pairs that build O, as in the 16-bit mode: the weights O / l then sum
        // to one exactly, and a row that sees a single key returns that key's V row bit for bit
        const bf16x2 ones = {(bf16_t)1.f, (bf16_t)1.f};
        u32x4 w[2];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][2 * e], cs, -mc));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][2 * e + 1], cs, -mc));
          const uint32_t pp = pack_bf16(p0, p1);
          l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pp), ones, l_run, false);
          w[e >> 2][e & 3] = pp;
        }
        pf[kb][0] = __builtin_bit_cast(bf16x8, w[0]);
        pf[kb][1] = __builtin_bit_cast(bf16x8, w[1]);
      }
    }

    // ---- O^T += V^T P^T.  MFMA step (kb,c) contracts tile rows 32kb+16c+{0..3,8..11}+4*g2 (+4 for the
    // second half of the lane's 8 values); the transposing read collects them from the row-major V tile.
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
      if (!act[kb]) continue;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
          oacc[db] = mfma_bf16(lds_read_transposed_swz(Vs + (32 * kb + 16 * c) * D, voff[db]), pf[kb][c], oacc[db]);
        }
    }
  };
  auto run_band = [&](auto fastc) {
    for (int tile = 0; tile < ntiles; tile += 2) {
      do_tile(tile, std::integral_constant<int, 0>{}, fastc);
      if (tile + 1 < ntiles) do_tile(tile + 1, std::integral_constant<int, 1>{}, fastc);
    }
  };
  // First with the softmax reference fixed at zero -- no maximum, no rescaling, nothing between the scores and
  // their exponentials: p = exp2(cs * s), exact as long as neither a probability nor a row sum leaves the range of
  // fp32 (any reference gives the same O / l).  Whether it did is known from the row sums at the end: a sum that is
  // infinite, not a number, or outside 2^-80 .. 2^80 sends the whole workgroup through its band again with the
  // running maximum of Eq. 1's usual online form (scores beyond +-55 / scale: not what attention logits look like).
  m_ref = 0.f;
  run_band(std::true_type{});
  float l_tot = sum_with_other_half(l_run);
  const bool out_of_range = s < n && !(l_tot > 0x1p-80f && l_tot < 0x1p80f);
  if (__syncthreads_or(out_of_range ? 1 : 0)) {
    m_ref = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    init_ring();
    __syncthreads();  // ring visible
    load_tile(0, 0);
    run_band(std::false_type{});
    l_tot = sum_with_other_half(l_run);
    __syncthreads();  // every wave is through its last tile (on the other path the vote above says so)
  }

  // ---- epilogue: normalise, transpose through LDS, scatter rows to their original positions
  const float inv_l = 1.f / l_tot;
  const size_t head_row0 = ((size_t)b * p.Hq + hq) * n;
  const size_t my_row = head_row0 + orig_q;  // this lane's output row (valid when s < n)
  if (p.LSE && g2 == 0 && s_w0 + c32 < n) p.LSE[my_row] = m_ref * p.scale + __logf(l_tot);
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] *= inv_l;

  // accumulator (db, 4mq..4mq+3) of a lane = elements 32db + 8mq + 4g2 .. +3 of its row
  bf16_t* Os = reinterpret_cast<bf16_t*>(smem) + wave * 32 * C::QSTR;
  bool area_free = true;  // the barrier that ended the tile loop has freed the staging area for its first use
  auto stage_and_store = [&](const f32x16* acc, void* dst_tensor) {
    if (!area_free) __syncthreads();  // the previous staging pass is stored
    area_free = false;
    int le = lane;  // the lane's staging address is formed here, from a copy the optimiser cannot trace back to
    asm volatile("" : "+v"(le));  // the prologue's (equal) one, which it would otherwise keep across the tile loop
    bf16_t* mine = Os + (le & 31) * C::QSTR + 4 * (le >> 5);
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int mq = 0; mq < 4; ++mq) {
        u32x2 w;
        w[0] = pack_bf16(acc[db][4 * mq + 0], acc[db][4 * mq + 1]);
        w[1] = pack_bf16(acc[db][4 * mq + 2], acc[db][4 * mq + 3]);
        *reinterpret_cast<u32x2*>(mine + 32 * db + 8 * mq) = w;
      }
    wave_lds_sync();  // the staging rows are this wave's own
    int dst[NP];
#pragma unroll
    for (int pass = 0; pass < NP; ++pass) dst[pass] = rowstash[wave * 32 + pass * C::WRPP + lane / C::CPR];
#pragma unroll
    for (int pass = 0; pass < NP; ++pass) {
      const int row = pass * C::WRPP + lane / C::CPR;
      if (s_w0 + row < n) {
        const size_t eoff = (head_row0 + dst[pass]) * D + chunk16 * 8;
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(Os + row * C::QSTR + chunk16 * 8),
                                    reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(dst_tensor) + eoff));
      }
    }
  };

  if (p.Y) stage_and_store(oacc, p.Y);
  if (GATED && p.gate_mode) {
    // Eq. 5: Y = sig(gamma_this) * Y_this + sig(gamma_other) * Y_other, formed in fp32: this branch enters
    // with its fp32 accumulators, the other one as the bf16 tensor it was stored as
    const size_t r = s_w0 + c32 < n ? my_row : head_row0;
    float ga = 0.f, gb = 0.f;
    if (!p.gate_per_dim) {
      ga = sigmoidf_exact(load_gate(p.gate_this, r, p.gate_f32));
      gb = sigmoidf_exact(load_gate(p.gate_other, r, p.gate_f32));
    }
    // the other branch's rows come in as whole rows through the staging area, the way this branch's leave (in the
    // accumulator layout a lane would ask memory for 8-byte pieces of 32 rows per instruction)
    {
      int src_row[NP];
#pragma unroll
      for (int pass = 0; pass < NP; ++pass) src_row[pass] = rowstash[wave * 32 + pass * C::WRPP + lane / C::CPR];
      u32x4 orow[NP];
#pragma unroll
      for (int pass = 0; pass < NP; ++pass)
        orow[pass] = load_row_chunk<D>(reinterpret_cast<const bf16_t*>(p.Y_other) + head_row0 * D, src_row[pass], chunk16);
      area_free = false;
      wave_lds_sync();  // the stores of this branch's rows, if there were any, have read the area
#pragma unroll
      for (int pass = 0; pass < NP; ++pass)
        *reinterpret_cast<u32x4*>(Os + (pass * C::WRPP + lane / C::CPR) * C::QSTR + chunk16 * 8) = orow[pass];
      wave_lds_sync();
    }
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int mq = 0; mq < 4; ++mq) {
        const size_t e0 = r * D + 32 * db + 8 * mq + 4 * g2;
        const u32x2 ob = *reinterpret_cast<const u32x2*>(Os + c32 * C::QSTR + 32 * db + 8 * mq + 4 * g2);
        const float o[4] = {bf16lo(ob[0]), bf16hi(ob[0]), bf16lo(ob[1]), bf16hi(ob[1])};
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          if (p.gate_per_dim) {
            ga = sigmoidf_exact(load_gate(p.gate_this, e0 + x, p.gate_f32));
            gb = sigmoidf_exact(load_gate(p.gate_other, e0 + x, p.gate_f32));
          }
          oacc[db][4 * mq + x] = ga * oacc[db][4 * mq + x] + gb * o[x];
        }
      }
    stage_and_store(oacc, p.Yout);
  }
}

template <int D>
hipError_t launch_t(const Pass& p, hipStream_t st) {
  // Query heads of a KV group that read K/V through the same permutation (or none) share a workgroup
  const bool shared_perm = !p.perm || p.perm_H == 1;
  const int hshift = !shared_perm ? 0 : (p.g % 4 == 0 ? 2 : (p.g % 2 == 0 ? 1 : 0));
  const int bm = BM >> hshift;
  const int num_qt = (p.n + bm - 1) / bm;
  const long total = (long)num_qt * (p.Hq >> hshift) * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(NT);
  // identity order with a one-sided linear window (plain causal SWA): the window already excludes every
  // later key, the causal test would only repeat it
  const bool window_is_causal = !p.perm && !p.win.circular && p.win.R == 0;
  const int mode = (!p.causal || window_is_causal) ? CAUSAL_NONE : (p.n <= 65535 ? CAUSAL_I16 : CAUSAL_I32);
#define SA_LAUNCH_FWD(PERM_, MODE_)                                                                              \
  do {                                                                                                            \
    if (gated) hipLaunchKernelGGL((fwd_mfma_bf16_kernel<D, PERM_, MODE_, true>), grid, block, 0, st, p, num_qt, total, hshift); \
    else hipLaunchKernelGGL((fwd_mfma_bf16_kernel<D, PERM_, MODE_, false>), grid, block, 0, st, p, num_qt, total, hshift);      \
  } while (0)
  const bool gated = p.gate_mode != 0;
  if (p.perm) {
    if (mode == CAUSAL_NONE) SA_LAUNCH_FWD(true, CAUSAL_NONE);
    else if (mode == CAUSAL_I16) SA_LAUNCH_FWD(true, CAUSAL_I16);
    else SA_LAUNCH_FWD(true, CAUSAL_I32);
  } else {
    if (mode == CAUSAL_NONE) SA_LAUNCH_FWD(false, CAUSAL_NONE);
    else if (mode == CAUSAL_I16) SA_LAUNCH_FWD(false, CAUSAL_I16);
    else SA_LAUNCH_FWD(false, CAUSAL_I32);
  }
#undef SA_LAUNCH_FWD
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_mfma_bf16(const Pass& p, hipStream_t st) {
  // geometry the kernel relies on
  if (p.n < 1 || p.B < 1 || p.Hq < 1 || p.Hkv < 1 || p.g * p.Hkv != p.Hq) return hipErrorInvalidValue;
  if (p.win.L < 0 || p.win.R < 0 || p.win.L >= p.n || p.win.R >= p.n) return hipErrorInvalidValue;
  if (p.win.circular && p.win.L + p.win.R + 1 > p.n) return hipErrorInvalidValue;
  if ((long)p.n * p.d * 2 >= (1L << 31)) return hipErrorNotSupported;  // 32-bit row offsets inside a head
  if (p.gate_mode && (!p.gate_this || !p.gate_other || !p.Y_other || !p.Yout)) return hipErrorInvalidValue;
  if (p.d == 64) return launch_t<64>(p, st);
  if (p.d == 128) return launch_t<128>(p, st);
  return hipErrorNotSupported;
}

}  // namespace sa
