// Gate projections of the dual-path layer on gfx950 matrix cores: Eq. 6 followed by Eq. 5
// (Alg. 2, "Gated Combination").
//
// Per token t = (b, i) the heads are concatenated to y_x[t] in R^{dm}, dm = Hq*d, and
//   logit_x[t,:] = W_x y_x[t],  g_x = sigmoid(logit_x),  Y[t,:] = g_sa * y_sa[t] + g_swa * y_swa[t].
// This is two dm x dm GEMMs over all tokens with an element-wise epilogue that needs the GEMM's own
// input at the output position.  One workgroup (4 waves, 2 x 2) owns 128 tokens x 128 output
// features and runs the two branches one after the other through the same LDS buffers, keeping the
// running sum in registers; a wave owns 64 x 64 as 2 x 2 blocks of v_mfma_f32_32x32x16_bf16, so
// every operand read from LDS feeds two matrix instructions.  Both operands have the contraction
// index contiguous in memory (the token's features inside a head, the weight's input features), so
// the tiles are staged row-major (+16 B row padding) and read with plain 16-byte loads.  The product
// is formed transposed (A operand = weight rows, B operand = token rows): a lane then owns one
// token and each accumulator quad four consecutive output features, i.e. 8 contiguous bytes of
// Y_x and Y.  The forward walks the contraction in rotated order, ending with the 128 input features
// that are the workgroup's own output features: the y_x values the epilogue multiplies the gates with
// are then the token tiles still lying in the two LDS buffers, and are not loaded a second time.
//
// Backward (given dY; g_x saved by the forward):
//   dz_x = dY * y_x * g_x * (1 - g_x)                     element-wise pass, rounded to bf16
//   dy_x = dY * g_x + W_x^T dz_x                          the forward kernel again: tokens = dz_x,
//                                                         weights = W_x^T (transposed once), epilogue = + dY * g_x
//   dW_x = sum_t dz_x[t] y_x[t]^T                         contraction over tokens: both operands are
//                                                         transposed on their way into LDS (4 x 8 register
//                                                         transposes), a workgroup owns 128 x 128 of dW for a
//                                                         chunk of tokens and adds it with fp32 atomics
#include "sa_common.h"
#include "sa_mfma.h"

namespace sa {
namespace {

constexpr int TM = 128;  // tokens per workgroup
constexpr int TN = 128;  // output features per workgroup
constexpr int TK = 64;   // contraction step
constexpr int GNT = 256;
constexpr int GSTR = TK + 8;                 // bf16 per LDS row
constexpr int TILE_BYTES = TM * GSTR * 2;    // one operand tile (TM == TN)
constexpr int GBUF_BYTES = 2 * TILE_BYTES;   // token tile | weight tile

struct GateProj {
  const void* Y_x[2];  // branch outputs [B,Hq,n,d]; Y_x[1] == nullptr: single path
  const void* W_x[2];  // [dm, dm] row-major, row = output feature
  void* G_x[2];        // optional: gate values sigmoid(logit) [B,Hq,n,d]
  void* Y;             // [B,Hq,n,d]
  const void* E1;      // backward-input mode: Y = acc + E1 * E2 (E1 = dY, E2 = g_x), both [B,Hq,n,d]
  const void* E2;
  int B, Hq, n, d;
};

enum { GP_FORWARD = 0, GP_BWD_INPUT = 1 };

template <int D, int MODE>
__global__ __launch_bounds__(GNT, 2) void gate_proj_fwd_bf16_kernel(const GateProj p, const int num_tt, const int num_ft,
                                                                    const long total_work) {
  __shared__ __attribute__((aligned(16))) char smem[2 * GBUF_BYTES];
  const long work = xcd_work_index(total_work);
  if (work < 0) return;
  // feature tiles vary fastest: consecutive workgroups read the same token tile
  const int ft = (int)(work % num_ft);
  long rest = work / num_ft;
  const int tt = (int)(rest % num_tt);
  const int b = (int)(rest / num_tt);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;  // token half, feature half of the workgroup tile
  const int g2 = lane >> 5, c32 = lane & 31;
  const int n = p.n, H = p.Hq, dm = H * D;
  const int i0 = tt * TM, o0 = ft * TN;
  const int nk = dm / TK;

  // loader: 128 rows x 8 chunks of 16 bytes per operand tile, 4 chunks per thread and operand
  const int lrow = tid >> 3, lchunk = tid & 7;  // rows lrow + 32*j
  u32x4 areg[4], wreg[4];
  // Forward: the two contraction steps that cover the workgroup's own 128 output features are taken last, so that
  // the token tiles left in the two buffers are the Y_x values Eq. 5 needs at the output positions (the epilogue
  // reads them from LDS instead of from memory).  The other steps keep their order: the workgroups that share a
  // token tile (the feature tiles of one token tile run side by side) then walk it nearly in step and find each
  // other's rows in L2 (fully rotated orders kept the whole tile of every group alive there: 4 x the fetches).
  const int own = MODE == GP_FORWARD ? o0 / TK : nk;  // (dm is a multiple of TN = 2 TK: nk >= 2)
  auto load_tiles = [&](const bf16_t* Yx, const bf16_t* Wx, int step) {
    const int kk = MODE != GP_FORWARD ? step : (step < nk - 2 ? (step < own ? step : step + 2) : own + step - (nk - 2));
    const int k0 = kk * TK, h = k0 / D, e0 = k0 % D;
    const bf16_t* abase = Yx + ((size_t)b * H + h) * n * (size_t)D + e0 + lchunk * 8;
    const bf16_t* wbase = Wx + (size_t)k0 + lchunk * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = lrow + 32 * j;
      areg[j] = *reinterpret_cast<const u32x4*>(abase + (size_t)min(i0 + row, n - 1) * D);
      wreg[j] = *reinterpret_cast<const u32x4*>(wbase + (size_t)(o0 + row) * dm);
    }
  };
  auto store_tiles = [&](int buf) {
    bf16_t* As = reinterpret_cast<bf16_t*>(smem + buf * GBUF_BYTES);
    bf16_t* Ws = reinterpret_cast<bf16_t*>(smem + buf * GBUF_BYTES + TILE_BYTES);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = lrow + 32 * j;
      *reinterpret_cast<u32x4*>(As + row * GSTR + lchunk * 8) = areg[j];
      *reinterpret_cast<u32x4*>(Ws + row * GSTR + lchunk * 8) = wreg[j];
    }
  };

  // running sum of Eq. 5: (fi, ti) = 32-feature block, 32-token block of the wave; accumulator
  // 4q + x of lane (g2, c32) is token 64wm + 32ti + c32, feature 64wn + 32fi + 8q + 4g2 + x
  f32x16 out[2][2];
#pragma unroll
  for (int fi = 0; fi < 2; ++fi)
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int i = 0; i < 16; ++i) out[fi][ti][i] = 0.f;

  // Output rows leave through a wave-private LDS area: the accumulator layout gives a lane 8-byte pieces of
  // 32 different rows, the staged copy lets 8 lanes write one full 128-byte piece of a row (non-temporal:
  // the outputs are written once).  Staging follows a workgroup barrier: the area lies on the two weight
  // tiles (waves 0, 1 on the first buffer's, waves 2, 3 on the second's), so the token tiles stay readable.
  constexpr int OSTR = 64 + 8;  // bf16 per staged row (64 features of one token + 16 B pad)
  static_assert(2 * 64 * OSTR * 2 == TILE_BYTES, "two waves' staging rows fill one weight tile");
  bf16_t* ostage = reinterpret_cast<bf16_t*>(smem + (wave >> 1) * GBUF_BYTES + TILE_BYTES) + (wave & 1) * 64 * OSTR;
  auto stage_put = [&](int fi, int ti, int q, u32x2 w) {
    *reinterpret_cast<u32x2*>(ostage + (32 * ti + c32) * OSTR + 32 * fi + 8 * q + 4 * g2) = w;
  };
  auto stage_flush = [&](bf16_t* dst) {
    wave_lds_sync();
    const int o = o0 + 64 * wn;  // first of the wave's 64 features: inside one head
    const size_t col = (size_t)(o % D) + (lane & 7) * 8;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int tl = pass * 8 + (lane >> 3);
      const int token = i0 + 64 * wm + tl;
      if (token < n) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(ostage + tl * OSTR + (lane & 7) * 8);
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst + (((size_t)b * H + o / D) * n + token) * D + col));
      }
    }
    wave_lds_sync();
  };

  // The other way round: the wave's 64 tokens x 64 features of a tensor come in as whole 128-byte pieces of rows
  // and are handed out in the accumulator layout (rows past n: the last row's values, never stored).
  auto stage_fetch_rows = [&](const bf16_t* src, u32x4* v) {
    const int o = o0 + 64 * wn;
    const size_t col = (size_t)(o % D) + (lane & 7) * 8;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int token = min(i0 + 64 * wm + pass * 8 + (lane >> 3), n - 1);
      v[pass] = *reinterpret_cast<const u32x4*>(src + (((size_t)b * H + o / D) * n + token) * D + col);
    }
  };
  auto stage_fetch_put = [&](const u32x4* v) {
#pragma unroll
    for (int pass = 0; pass < 8; ++pass)
      *reinterpret_cast<u32x4*>(ostage + (pass * 8 + (lane >> 3)) * OSTR + (lane & 7) * 8) = v[pass];
    wave_lds_sync();
  };
  auto stage_get = [&](int fi, int ti, int q) -> u32x2 {
    return *reinterpret_cast<const u32x2*>(ostage + (32 * ti + c32) * OSTR + 32 * fi + 8 * q + 4 * g2);
  };

  const int branches = p.Y_x[1] ? 2 : 1;
  for (int x = 0; x < branches; ++x) {
    const bf16_t* Yx = reinterpret_cast<const bf16_t*>(p.Y_x[x]);
    const bf16_t* Wx = reinterpret_cast<const bf16_t*>(p.W_x[x]);
    f32x16 acc[2][2];
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[fi][ti][i] = 0.f;

    __syncthreads();  // the previous branch is done with both buffers
    load_tiles(Yx, Wx, 0);
    store_tiles(0);
    if (nk > 1) load_tiles(Yx, Wx, 1);
    for (int kk = 0; kk < nk; ++kk) {
      const int buf = kk & 1;
      __syncthreads();  // buffer `buf` is complete; everyone is done with the other one
      if (kk + 1 < nk) {
        store_tiles(buf ^ 1);
        if (kk + 2 < nk) load_tiles(Yx, Wx, kk + 2);
      }
      const bf16_t* As = reinterpret_cast<const bf16_t*>(smem + buf * GBUF_BYTES) + (64 * wm + c32) * GSTR + 8 * g2;
      const bf16_t* Ws = reinterpret_cast<const bf16_t*>(smem + buf * GBUF_BYTES + TILE_BYTES) + (64 * wn + c32) * GSTR + 8 * g2;
#pragma unroll
      for (int ks = 0; ks < TK / 16; ++ks) {
        bf16x8 fa[2], fb[2];
#pragma unroll
        for (int fi = 0; fi < 2; ++fi) fa[fi] = *reinterpret_cast<const bf16x8*>(Ws + 32 * fi * GSTR + 16 * ks);
#pragma unroll
        for (int ti = 0; ti < 2; ++ti) fb[ti] = *reinterpret_cast<const bf16x8*>(As + 32 * ti * GSTR + 16 * ks);
#pragma unroll
        for (int fi = 0; fi < 2; ++fi)
#pragma unroll
          for (int ti = 0; ti < 2; ++ti) acc[fi][ti] = mfma_bf16(fa[fi], fb[ti], acc[fi][ti]);
      }
    }

    // Eq. 6 / Eq. 5 for this branch: out += sigmoid(logit) * Y_x at the same (token, feature)
    // (backward-input mode: out = product + dY * g_x)
    bf16_t* Gx = reinterpret_cast<bf16_t*>(p.G_x[x]);
    const bf16_t* E1 = reinterpret_cast<const bf16_t*>(p.E1);
    const bf16_t* E2 = reinterpret_cast<const bf16_t*>(p.E2);
    // step nk-2 left features o0 .. o0+63 of the token tile in its buffer, step nk-1 the next 64: this wave's 64
    // features are in the buffer of step nk-2+wn (the output staging area below lies on the weight tiles only)
    const bf16_t* Ay = reinterpret_cast<const bf16_t*>(smem + ((nk - 2 + wn) & 1) * GBUF_BYTES) + (64 * wm + c32) * GSTR + 4 * g2;
    if (MODE == GP_FORWARD && Gx) __syncthreads();  // every wave has read its last operands: the area is free
    u32x2 e1[2][2][4];
    if (MODE == GP_BWD_INPUT) {
      // dY and g_x at the output positions: whole rows through the staging area (the accumulator layout would
      // ask memory for 8-byte pieces of 32 rows per instruction)
      u32x4 r1[8], r2[8];
      stage_fetch_rows(E1, r1);
      stage_fetch_rows(E2, r2);
      __syncthreads();  // every wave has read its last operands: the area is free
      stage_fetch_put(r1);
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int fi = 0; fi < 2; ++fi)
#pragma unroll
          for (int q = 0; q < 4; ++q) e1[ti][fi][q] = stage_get(fi, ti, q);
      wave_lds_sync();
      stage_fetch_put(r2);
    }
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
      const int token = i0 + 64 * wm + 32 * ti + c32;
      const bool live = token < n;
      const int tk = live ? token : n - 1;
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int o = o0 + 64 * wn + 32 * fi + 8 * q + 4 * g2;  // first of four consecutive features
          const size_t at = (((size_t)b * H + o / D) * n + tk) * D + o % D;
          if (MODE == GP_FORWARD) {
            const u32x2 y = *reinterpret_cast<const u32x2*>(Ay + 32 * ti * GSTR + 32 * fi + 8 * q);
            const float yv[4] = {bf16lo(y[0]), bf16hi(y[0]), bf16lo(y[1]), bf16hi(y[1])};
            float gv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              gv[e] = sigmoidf_rcp(acc[fi][ti][4 * q + e]);
              out[fi][ti][4 * q + e] = fmaf(gv[e], yv[e], out[fi][ti][4 * q + e]);
            }
            if (Gx) {
              u32x2 w;
              w[0] = pack_bf16(gv[0], gv[1]);
              w[1] = pack_bf16(gv[2], gv[3]);
              stage_put(fi, ti, q, w);
            }
          } else {
            const u32x2 a = e1[ti][fi][q], c = stage_get(fi, ti, q);
            out[fi][ti][4 * q + 0] = fmaf(bf16lo(a[0]), bf16lo(c[0]), acc[fi][ti][4 * q + 0]);
            out[fi][ti][4 * q + 1] = fmaf(bf16hi(a[0]), bf16hi(c[0]), acc[fi][ti][4 * q + 1]);
            out[fi][ti][4 * q + 2] = fmaf(bf16lo(a[1]), bf16lo(c[1]), acc[fi][ti][4 * q + 2]);
            out[fi][ti][4 * q + 3] = fmaf(bf16hi(a[1]), bf16hi(c[1]), acc[fi][ti][4 * q + 3]);
          }
        }
    }
    if (MODE == GP_FORWARD && Gx) stage_flush(Gx);
  }

  __syncthreads();  // every wave has read its last operands (or flushed its last gate rows): the area is free
#pragma unroll
  for (int ti = 0; ti < 2; ++ti)
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        u32x2 w;
        w[0] = pack_bf16(out[fi][ti][4 * q + 0], out[fi][ti][4 * q + 1]);
        w[1] = pack_bf16(out[fi][ti][4 * q + 2], out[fi][ti][4 * q + 3]);
        stage_put(fi, ti, q, w);
      }
  stage_flush(reinterpret_cast<bf16_t*>(p.Y));
}


// dz = dY * y * g * (1 - g), rounded to bf16; 8 elements per thread.
__global__ __launch_bounds__(256) void gate_dz_bf16_kernel(const uint16_t* __restrict__ dY, const uint16_t* __restrict__ Yx,
                                                            const uint16_t* __restrict__ Gx, uint16_t* __restrict__ dz,
                                                            const size_t vecs) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < vecs; i += stride) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(dY + 8 * i), y = *reinterpret_cast<const u32x4*>(Yx + 8 * i);
    const u32x4 g = *reinterpret_cast<const u32x4*>(Gx + 8 * i);
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float gl = bf16lo(g[e]), gh = bf16hi(g[e]);
      o[e] = pack_bf16(bf16lo(a[e]) * bf16lo(y[e]) * gl * (1.f - gl), bf16hi(a[e]) * bf16hi(y[e]) * gh * (1.f - gh));
    }
    *reinterpret_cast<u32x4*>(dz + 8 * i) = o;
  }
}

// Wt[k][o] = W[o][k] for a square bf16 matrix (dm a multiple of 64): 64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ Wt, const int dm) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int e = threadIdx.x; e < 64 * 64; e += 256) tile[e / 64][e % 64] = W[(size_t)(r0 + e / 64) * dm + c0 + e % 64];
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 64; e += 256) Wt[(size_t)(c0 + e / 64) * dm + r0 + e % 64] = tile[e % 64][e / 64];
}

// dW[o][k] += sum over a chunk of tokens of dz[t][o] * y[t][k].  Workgroup = 128 x 128 of dW, 4 waves
// as 2 x 2.  The contraction runs over tokens, which is the slow index of both operands in memory, so
// both tiles are brought in as they lie ([token][128 features], by direct global-to-LDS loads, unpadded
// rows with swizzled 16-byte chunks) and both operands are read with the transposing LDS read: a lane
// gets the same 8 tokens of one feature column for the A operand (dz^T) and the B operand (y).
// Steps of 32 tokens, four buffers, three steps in flight.  Tokens past the chunk's end are zeroed in
// the dz tile after it has landed.
constexpr int WCHUNK = 4096;  // tokens per workgroup
constexpr int WSTEP = 32;
constexpr int WSTAGES = 4;
constexpr int WTILE_BYTES = WSTEP * 128 * 2;  // one operand, one step
constexpr int WSTAGE_BYTES = 2 * WTILE_BYTES;
constexpr int WLOADS_PER_STAGE = 4;           // instructions per thread: 2 rows of 16 tokens x 2 operands

template <int D>
__global__ __launch_bounds__(GNT, 2) void gate_dw_bf16_kernel(const bf16_t* __restrict__ dz, const bf16_t* __restrict__ Yx,
                                                               float* __restrict__ dW, const int B, const int H, const int n,
                                                               const int num_ft, const int chunks_per_b, const long total_work) {
  __shared__ __attribute__((aligned(16))) char smem[WSTAGES * WSTAGE_BYTES];
  const long work = xcd_work_index(total_work);
  if (work < 0) return;
  const int kt = (int)(work % num_ft);  // input-feature tile (columns of dW)
  long rest = work / num_ft;
  const int ot = (int)(rest % num_ft);  // output-feature tile (rows of dW)
  rest /= num_ft;
  const int ch = (int)(rest % chunks_per_b);
  const int b = (int)(rest / chunks_per_b);
  const int dm = H * D;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = wave & 1, wk = wave >> 1;
  const int g2 = lane >> 5, c32 = lane & 31;
  const int t_begin = ch * WCHUNK, t_end = min(t_begin + WCHUNK, n);
  const int nsteps = (t_end - t_begin + WSTEP - 1) / WSTEP;

  // loader: one instruction of a wave fills 4 token rows (256 bytes each) of a tile; the lane delivers
  // physical chunk lane % 16 of token row wave * 4 + lane / 16 (+16 for the second instruction), i.e.
  // fetches the logical chunk (lane % 16) ^ swz(row): 8 features of one head
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const int ld_row = wave * 4 + (lane >> 4);
  const int ld_feat = 8 * ((lane & 15) ^ swz<128>(ld_row));
  auto feature_offset = [&](int f) -> uint32_t {  // bytes from the batch's first element to (token 0, feature f)
    return (uint32_t)(((size_t)(f / D) * n * D + f % D) * 2);
  };
  const bf16_t* zb = dz + (size_t)b * H * n * D;
  const bf16_t* yb = Yx + (size_t)b * H * n * D;
  const uint32_t zfeat = feature_offset(ot * 128 + ld_feat), yfeat = feature_offset(kt * 128 + ld_feat);
  auto request_step = [&](int st) {  // steps past the last one fetch its rows again and are never used
    const int buf = st & (WSTAGES - 1);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int token = min(t_begin + st * WSTEP + 16 * j + ld_row, t_end - 1);
      const uint32_t trow = (uint32_t)token * (uint32_t)(D * 2);
      const uint32_t dst = lds0 + buf * WSTAGE_BYTES + (16 * j + wave * 4) * 256;
      load_to_lds_16(zb, zfeat + trow, dst);
      load_to_lds_16(yb, yfeat + trow, dst + WTILE_BYTES);
    }
  };

  int troff[4][2];
  swizzled_tr_offsets<128>(lane, troff);

  f32x16 acc[2][2];
#pragma unroll
  for (int oi = 0; oi < 2; ++oi)
#pragma unroll
    for (int ki = 0; ki < 2; ++ki)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[oi][ki][i] = 0.f;

  request_step(0);
  request_step(1);
  request_step(2);
  for (int st = 0; st < nsteps; ++st) {
    const int buf = st & (WSTAGES - 1);
    // all but the two youngest steps of this wave have landed; after the barrier step st is visible and
    // everyone is done with the buffer of step st - 1, which step st + 3 may now overwrite
    __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * WLOADS_PER_STAGE));  // vmcnt(8)
    __syncthreads();
    request_step(st + 3);
    bf16_t* Zt = reinterpret_cast<bf16_t*>(smem + buf * WSTAGE_BYTES);
    const bf16_t* Yt = reinterpret_cast<const bf16_t*>(smem + buf * WSTAGE_BYTES + WTILE_BYTES);
    if (t_begin + (st + 1) * WSTEP > t_end) {  // ragged last step: tokens past the end contribute zeros
      const int row = tid >> 3;
      if (t_begin + st * WSTEP + row >= t_end) {
        u32x4* r = reinterpret_cast<u32x4*>(Zt + row * 128 + (tid & 7) * 16);
        r[0] = u32x4{0u, 0u, 0u, 0u};
        r[1] = u32x4{0u, 0u, 0u, 0u};
      }
      __syncthreads();
    }
#pragma unroll
    for (int ks = 0; ks < WSTEP / 16; ++ks) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int oi = 0; oi < 2; ++oi) fa[oi] = lds_read_transposed_swz(Zt + 16 * ks * 128, troff[2 * wo + oi]);
#pragma unroll
      for (int ki = 0; ki < 2; ++ki) fb[ki] = lds_read_transposed_swz(Yt + 16 * ks * 128, troff[2 * wk + ki]);
#pragma unroll
      for (int oi = 0; oi < 2; ++oi)
#pragma unroll
        for (int ki = 0; ki < 2; ++ki) acc[oi][ki] = mfma_bf16(fa[oi], fb[ki], acc[oi][ki]);
    }
  }
  wait_all_loads();  // the surplus steps requested near the end
  // accumulator 4q + x of lane (g2, c32): row o = 64wo + 32oi + 8q + 4g2 + x, column k = 64wk + 32ki + c32
#pragma unroll
  for (int oi = 0; oi < 2; ++oi)
#pragma unroll
    for (int ki = 0; ki < 2; ++ki)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int o = ot * 128 + 64 * wo + 32 * oi + 8 * (i / 4) + 4 * g2 + (i % 4);
        const int k = kt * 128 + 64 * wk + 32 * ki + c32;
        unsafeAtomicAdd(dW + (size_t)o * dm + k, acc[oi][ki][i]);  // hardware fp32 add, device memory
      }
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, const size_t pairs) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < pairs; i += stride) {
    const f32x2 v = *reinterpret_cast<const f32x2*>(src + 2 * i);
    *reinterpret_cast<uint32_t*>(dst + 2 * i) = pack_bf16(v[0], v[1]);
  }
}

template <int MODE>
hipError_t launch_gemm(const GateProj& p, hipStream_t st) {
  const long dm = (long)p.Hq * p.d;
  const int num_tt = (p.n + TM - 1) / TM, num_ft = (int)(dm / TN);
  const long total = (long)num_tt * num_ft * p.B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  if (p.d == 64) hipLaunchKernelGGL((gate_proj_fwd_bf16_kernel<64, MODE>), dim3((unsigned)blocks), dim3(GNT), 0, st, p, num_tt, num_ft, total);
  else hipLaunchKernelGGL((gate_proj_fwd_bf16_kernel<128, MODE>), dim3((unsigned)blocks), dim3(GNT), 0, st, p, num_tt, num_ft, total);
  return hipGetLastError();
}

unsigned capped_blocks(size_t items, size_t per_block) {
  const size_t want = (items + per_block - 1) / per_block;
  return (unsigned)(want < 1 ? 1 : (want > 65536 ? 65536 : want));
}

}  // namespace

hipError_t launch_gate_proj_fwd_bf16(int B, int Hq, int n, int d, const void* Y_sa, const void* Y_swa, const void* W_sa,
                                     const void* W_swa, void* Y, void* G_sa, void* G_swa, hipStream_t st) {
  if (B < 1 || Hq < 1 || n < 1 || !Y_sa || !W_sa || !Y) return hipErrorInvalidValue;
  if ((Y_swa == nullptr) != (W_swa == nullptr)) return hipErrorInvalidValue;
  if (!(d == 64 || d == 128)) return hipErrorNotSupported;
  const long dm = (long)Hq * d;
  if (dm % TN != 0 || dm % TK != 0) return hipErrorNotSupported;  // whole feature tiles only
  GateProj p = {};
  p.Y_x[0] = Y_sa; p.Y_x[1] = Y_swa;
  p.W_x[0] = W_sa; p.W_x[1] = W_swa;
  p.G_x[0] = G_sa; p.G_x[1] = G_swa;
  p.Y = Y;
  p.B = B; p.Hq = Hq; p.n = n; p.d = d;
  return launch_gemm<GP_FORWARD>(p, st);
}

size_t gate_proj_bwd_workspace_bytes(int B, int Hq, int n, int d, bool dual) {
  const size_t dm = (size_t)Hq * d, act = (size_t)B * Hq * n * d;
  const size_t per_branch = act * 2 /* dz bf16 */ + dm * dm * 2 /* W^T bf16 */ + dm * dm * 4 /* dW fp32 */;
  return (dual ? 2 : 1) * ((per_branch + 255) / 256 * 256);
}

// One branch: dz, W^T, dy_x = dY * g_x + dz W_x, dW_x = dz^T y_x.
static hipError_t gate_proj_bwd_branch(int B, int Hq, int n, int d, const void* Yx, const void* Wx, const void* Gx,
                                       const void* dY, void* dYx, void* dWx, char* ws, hipStream_t st) {
  const size_t dm = (size_t)Hq * d, act = (size_t)B * Hq * n * d;
  uint16_t* dz = reinterpret_cast<uint16_t*>(ws);
  uint16_t* Wt = reinterpret_cast<uint16_t*>(ws + act * 2);
  float* dWf = reinterpret_cast<float*>(ws + act * 2 + dm * dm * 2);
  hipLaunchKernelGGL(gate_dz_bf16_kernel, dim3(capped_blocks(act / 8, 256)), dim3(256), 0, st,
                     reinterpret_cast<const uint16_t*>(dY), reinterpret_cast<const uint16_t*>(Yx),
                     reinterpret_cast<const uint16_t*>(Gx), dz, act / 8);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)(dm / 64), (unsigned)(dm / 64)), dim3(256), 0, st,
                     reinterpret_cast<const uint16_t*>(Wx), Wt, (int)dm);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  GateProj p = {};
  p.Y_x[0] = dz; p.W_x[0] = Wt;
  p.Y = dYx; p.E1 = dY; p.E2 = Gx;
  p.B = B; p.Hq = Hq; p.n = n; p.d = d;
  e = launch_gemm<GP_BWD_INPUT>(p, st);
  if (e != hipSuccess) return e;
  e = launch_fill_zero(dWf, dm * dm * 4, st);
  if (e != hipSuccess) return e;
  const int num_ft = (int)(dm / 128), chunks = (n + WCHUNK - 1) / WCHUNK;
  const long total = (long)num_ft * num_ft * chunks * B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  if (d == 64) hipLaunchKernelGGL(gate_dw_bf16_kernel<64>, dim3((unsigned)blocks), dim3(GNT), 0, st, reinterpret_cast<const bf16_t*>(dz),
                                  reinterpret_cast<const bf16_t*>(Yx), dWf, B, Hq, n, num_ft, chunks, total);
  else hipLaunchKernelGGL(gate_dw_bf16_kernel<128>, dim3((unsigned)blocks), dim3(GNT), 0, st, reinterpret_cast<const bf16_t*>(dz),
                          reinterpret_cast<const bf16_t*>(Yx), dWf, B, Hq, n, num_ft, chunks, total);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(capped_blocks(dm * dm / 2, 256)), dim3(256), 0, st, dWf,
                     reinterpret_cast<uint16_t*>(dWx), dm * dm / 2);
  return hipGetLastError();
}

hipError_t launch_gate_proj_bwd_bf16(int B, int Hq, int n, int d, const void* Y_sa, const void* Y_swa, const void* W_sa,
                                     const void* W_swa, const void* G_sa, const void* G_swa, const void* dY, void* dY_sa,
                                     void* dY_swa, void* dW_sa, void* dW_swa, void* ws, hipStream_t st) {
  if (B < 1 || Hq < 1 || n < 1 || !Y_sa || !W_sa || !G_sa || !dY || !dY_sa || !dW_sa || !ws) return hipErrorInvalidValue;
  const bool dual = Y_swa != nullptr;
  if (dual != (W_swa != nullptr) || dual != (G_swa != nullptr) || dual != (dY_swa != nullptr) || dual != (dW_swa != nullptr))
    return hipErrorInvalidValue;
  if (!(d == 64 || d == 128)) return hipErrorNotSupported;
  const long dm = (long)Hq * d;
  if (dm % 128 != 0) return hipErrorNotSupported;
  if ((size_t)dm * n * 2 >= ((size_t)1 << 32)) return hipErrorNotSupported;  // 32-bit byte offsets inside a batch
  char* base = reinterpret_cast<char*>(ws);
  hipError_t e = gate_proj_bwd_branch(B, Hq, n, d, Y_sa, W_sa, G_sa, dY, dY_sa, dW_sa, base, st);
  if (e != hipSuccess || !dual) return e;
  const size_t half = gate_proj_bwd_workspace_bytes(B, Hq, n, d, false);
  return gate_proj_bwd_branch(B, Hq, n, d, Y_swa, W_swa, G_swa, dY, dY_swa, dW_swa, base + half, st);
}

}  // namespace sa
