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
// Y_x and Y.
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
  int B, Hq, n, d;
};

template <int D>
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
  auto load_tiles = [&](const bf16_t* Yx, const bf16_t* Wx, int kk) {
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
    bf16_t* Gx = reinterpret_cast<bf16_t*>(p.G_x[x]);
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
          const u32x2 y = *reinterpret_cast<const u32x2*>(Yx + at);
          const float yv[4] = {bf16lo(y[0]), bf16hi(y[0]), bf16lo(y[1]), bf16hi(y[1])};
          float gv[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            gv[e] = sigmoidf_exact(acc[fi][ti][4 * q + e]);
            out[fi][ti][4 * q + e] = fmaf(gv[e], yv[e], out[fi][ti][4 * q + e]);
          }
          if (Gx && live) {
            u32x2 w;
            w[0] = pack_bf16(gv[0], gv[1]);
            w[1] = pack_bf16(gv[2], gv[3]);
            *reinterpret_cast<u32x2*>(Gx + at) = w;
          }
        }
    }
  }

  bf16_t* Yo = reinterpret_cast<bf16_t*>(p.Y);
#pragma unroll
  for (int ti = 0; ti < 2; ++ti) {
    const int token = i0 + 64 * wm + 32 * ti + c32;
    if (token >= n) continue;
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int o = o0 + 64 * wn + 32 * fi + 8 * q + 4 * g2;
        const size_t at = (((size_t)b * H + o / D) * n + token) * D + o % D;
        u32x2 w;
        w[0] = pack_bf16(out[fi][ti][4 * q + 0], out[fi][ti][4 * q + 1]);
        w[1] = pack_bf16(out[fi][ti][4 * q + 2], out[fi][ti][4 * q + 3]);
        *reinterpret_cast<u32x2*>(Yo + at) = w;
      }
  }
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
  const int num_tt = (n + TM - 1) / TM, num_ft = (int)(dm / TN);
  const long total = (long)num_tt * num_ft * B;
  const long blocks = xcd_grid_blocks(total);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  if (d == 64) hipLaunchKernelGGL(gate_proj_fwd_bf16_kernel<64>, dim3((unsigned)blocks), dim3(GNT), 0, st, p, num_tt, num_ft, total);
  else hipLaunchKernelGGL(gate_proj_fwd_bf16_kernel<128>, dim3((unsigned)blocks), dim3(GNT), 0, st, p, num_tt, num_ft, total);
  return hipGetLastError();
}

}  // namespace sa
