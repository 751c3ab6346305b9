// Matrix-core building blocks shared by the bf16 forward and backward kernels (gfx950).
#pragma once

#include "sa_device.h"

namespace sa {

constexpr int NXCD = 8;  // workgroup ids are dealt round-robin to the 8 XCDs

typedef short s16x8 __attribute__((ext_vector_type(8)));

// D = A(32x16) * B(16x32) + C.  Lane l = 32*g + r holds A[r][8g..8g+7], B[8g..8g+7][r] and the
// accumulators C[8*(i/4) + 4g + i%4][r], i = 0..15.
__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// The same product written as an instruction, with the accumulator pinned to the vector half of the register
// file.  A kernel that is allowed more than 256 registers per lane gets matrix results in the accumulator half
// by default, and every vector instruction that uses them (scores, probabilities) then needs a copy first.
// The compiler does not know what the statement is: the wait states between the last product of a chain and the
// first vector instruction that reads its result are supplied by matrix_results_to_vector().
__device__ __forceinline__ void mfma_bf16_v_first(const bf16x8 a, const bf16x8 b, f32x16& acc) {  // acc = A B
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_bf16_v(const bf16x8 a, const bf16x8 b, f32x16& acc) {  // acc += A B
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void matrix_results_to_vector(f32x16& x, f32x16& y) {
  asm volatile("s_nop 11" : "+v"(x), "+v"(y));
}

// Transposing LDS read (ds_read_b64_tr_b16): within a group of 16 lanes, lane i receives element
// (i % 4) of the 8-byte words addressed by lanes i/4, i/4+4, i/4+8, i/4+12 of the group.
__device__ __forceinline__ s16x4 lds_read_tr16(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

// A operand X^T (32 columns of X starting at col0, contraction over 16 rows of X) for a row-major
// LDS tile X[row][stride]: the contraction rows are row0 + {0..3, 8..11} + 4*g (lanes' first four
// values) and +4 more (second four), which is exactly where the accumulators of a preceding
// 32x32 product keep the values that serve as the B operand (elements 8c..8c+7 of the lane).
__device__ __forceinline__ bf16x8 lds_read_transposed_a(const bf16_t* tile, int stride, int row0, int col0, int lane) {
  const int G = lane >> 4, j16 = lane & 15;
  const bf16_t* base = tile + (row0 + 4 * (G >> 1) + (j16 >> 2)) * stride + col0 + 16 * (G & 1) + 4 * (j16 & 3);
  const s16x4 lo = lds_read_tr16(base);
  const s16x4 hi = lds_read_tr16(base + 8 * stride);
  const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, a);
}

// K and V tiles lie in LDS as they lie in memory (row after row, no padding: that is how the direct
// global-to-LDS loads deliver them), with the 16-byte chunks of a row permuted by an XOR with swz(row)
// so that the two read patterns are conflict-free: 16 rows x the same chunk (K operand, ds_read_b128)
// and 4 rows x 4 consecutive chunks (V operand, transposing 8-byte reads).
template <int D>
__device__ __forceinline__ int swz(int row) {
  return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

// 16 bytes per lane from global memory (scalar base + 32-bit lane offset) straight into LDS at
// lds_byte_addr + 16 * lane.  The address travels in M0 and must be wave-uniform; it is handed to the
// statement as a register operand, so the compiler knows that M0 is written here (the no-op covers the wait
// state an LDS-DMA instruction needs after a scalar write of M0).  The compiler does not see the load
// itself: it is waited for with an explicit s_waitcnt vmcnt before the barrier that publishes the tile.
__device__ __forceinline__ void load_to_lds_16(const void* base, uint32_t lane_byte_offset, uint32_t lds_byte_addr) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_byte_addr);
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_byte_offset), "s"(base), "{m0}"(m0) : "memory");
}
__device__ __forceinline__ void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only

// Element offsets, inside a swizzled tile of D-element rows, of a lane's operand reads (the rows of the
// 32-row block are added by the caller):
//   row operand kk (plain 16-byte read): row c32 of the block, logical chunk 2 kk + g2;
//   transposed operand (db, half): the transposing read of lane (G = lane / 16, j = lane % 16) takes 8
//   bytes of row 4 (G / 2) + j / 4 (+8 for the second half) of a 16-row block at columns
//   32 db + 16 (G % 2) + 4 (j % 4) .. +3.
template <int D>
__device__ __forceinline__ void swizzled_row_offsets(int lane, int* off) {
  const int g2 = lane >> 5, c32 = lane & 31;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) off[kk] = c32 * D + 8 * ((2 * kk + g2) ^ swz<D>(c32));
}
template <int D>
__device__ __forceinline__ void swizzled_tr_offsets(int lane, int (*off)[2]) {
  const int G = lane >> 4, j16 = lane & 15;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int row = 4 * (G >> 1) + (j16 >> 2) + 8 * hf;
      const int col = 32 * db + 16 * (G & 1) + 4 * (j16 & 3);
      off[db][hf] = row * D + 8 * ((col >> 3) ^ swz<D>(row)) + (col & 7);
    }
}
// A operand X^T for 16 contraction rows starting at `rows16` (a multiple of 16 rows into a swizzled tile):
// the contraction rows are {0..3, 8..11} + 4*g (first four values of the lane) and +4 more (second four),
// which is where the accumulators of a preceding 32x32 product keep the values that serve as B operand.
__device__ __forceinline__ bf16x8 lds_read_transposed_swz(const bf16_t* rows16, const int* off2) {
  const s16x4 lo = lds_read_tr16(rows16 + off2[0]), hi = lds_read_tr16(rows16 + off2[1]);
  const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, a);
}

// RoPE (RoFormer Sec. 3.2.2) of one row held as MFMA operand fragments: lane group g2 holds elements
// 16kk + 8*g2 .. +7 of the row in f[kk], so both members of a pair are the lane's own -- (x[i], x[i + D/2]) sit
// in fragments kk and kk + D/32, (x[2i], x[2i+1]) next to each other.  trow: the (cos, sin) of the row's
// position, D/2 pairs.  The rotated values are rounded to bf16.
template <int D>
__device__ __forceinline__ void rope_row_fragments(bf16x8* f, const float2* trow, int g2, int interleaved) {
  if (!interleaved) {
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      const float4* tp = reinterpret_cast<const float4*>(trow + 16 * kk + 8 * g2);
      const u32x4 a = __builtin_bit_cast(u32x4, f[kk]), b = __builtin_bit_cast(u32x4, f[kk + D / 32]);
      u32x4 ra, rb;
#pragma unroll
      for (int m = 0; m < 4; ++m) {  // dword m = elements 2m, 2m+1 of the fragment
        const float4 t = tp[m];      // (cos, sin) of pairs 2m and 2m+1
        const float a0 = bf16lo(a[m]), a1 = bf16hi(a[m]), b0 = bf16lo(b[m]), b1 = bf16hi(b[m]);
        ra[m] = pack_bf16(a0 * t.x - b0 * t.y, a1 * t.z - b1 * t.w);
        rb[m] = pack_bf16(a0 * t.y + b0 * t.x, a1 * t.w + b1 * t.z);
      }
      f[kk] = __builtin_bit_cast(bf16x8, ra);
      f[kk + D / 32] = __builtin_bit_cast(bf16x8, rb);
    }
  } else {
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const float4* tp = reinterpret_cast<const float4*>(trow + 8 * kk + 4 * g2);
      const u32x4 a = __builtin_bit_cast(u32x4, f[kk]);
      u32x4 ra;
#pragma unroll
      for (int m = 0; m < 2; ++m) {  // dwords 2m, 2m+1 = pairs 2m, 2m+1 of the fragment
        const float4 t = tp[m];
        const float x0 = bf16lo(a[2 * m]), y0 = bf16hi(a[2 * m]);
        const float x1 = bf16lo(a[2 * m + 1]), y1 = bf16hi(a[2 * m + 1]);
        ra[2 * m] = pack_bf16(x0 * t.x - y0 * t.y, x0 * t.y + y0 * t.x);
        ra[2 * m + 1] = pack_bf16(x1 * t.z - y1 * t.w, x1 * t.w + y1 * t.z);
      }
      f[kk] = __builtin_bit_cast(bf16x8, ra);
    }
  }
}

// The transpose of that rotation (turn by the negative angle: the backward of RoPE) on a row held as transposed
// accumulators: accumulator 4*mq + x of block db of lane group g2 is element 32 db + 8 mq + 4 g2 + x of the
// lane's row, so again both members of a pair are the lane's own -- elements i and i + D/2 in blocks db and
// db + D/64, elements 2i and 2i+1 in accumulators x = 0, 1 and 2, 3.  In fp32, in place.
template <int D>
__device__ __forceinline__ void rope_transpose_accumulators(f32x16* acc, const float2* trow, int g2, int interleaved) {
  if (!interleaved) {
#pragma unroll
    for (int db = 0; db < D / 64; ++db)
#pragma unroll
      for (int mq = 0; mq < 4; ++mq) {
        const float4* tp = reinterpret_cast<const float4*>(trow + 32 * db + 8 * mq + 4 * g2);
        const float4 t01 = tp[0], t23 = tp[1];  // (cos, sin) of pairs x = 0, 1 and x = 2, 3
        const float c[4] = {t01.x, t01.z, t23.x, t23.z}, sn[4] = {t01.y, t01.w, t23.y, t23.w};
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const float a = acc[db][4 * mq + x], b = acc[db + D / 64][4 * mq + x];
          acc[db][4 * mq + x] = a * c[x] + b * sn[x];
          acc[db + D / 64][4 * mq + x] = b * c[x] - a * sn[x];
        }
      }
  } else {
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int mq = 0; mq < 4; ++mq) {
        const float4 t = *reinterpret_cast<const float4*>(trow + 16 * db + 4 * mq + 2 * g2);  // pairs of x = 0,1 and 2,3
        const float a0 = acc[db][4 * mq + 0], b0 = acc[db][4 * mq + 1], a1 = acc[db][4 * mq + 2], b1 = acc[db][4 * mq + 3];
        acc[db][4 * mq + 0] = a0 * t.x + b0 * t.y;
        acc[db][4 * mq + 1] = b0 * t.x - a0 * t.y;
        acc[db][4 * mq + 2] = a1 * t.z + b1 * t.w;
        acc[db][4 * mq + 3] = b1 * t.z - a1 * t.w;
      }
  }
}

// Pack accumulators 8c..8c+7 of a lane as a bf16 B operand.
__device__ __forceinline__ bf16x8 pack_b_operand(const float* v8) {
  u32x4 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = pack_bf16(v8[2 * e], v8[2 * e + 1]);
  return __builtin_bit_cast(bf16x8, w);
}

// Position (in units of 4 slots) of the 4-slot group u of a streamed tile inside a row of its
// transposed LDS copy.  Accumulator i = 8c + 4h + x of lane group g holds tile row
// 32kb + 16c + 8h + 4g + x; storing that row at 32kb + 16c + 8g + 4h + x makes the 8 values a lane
// needs as A operand of MFMA step (kb, c) one contiguous 16-byte read.
__device__ __forceinline__ int transposed_pos4(int u) {
  return (u & ~3) | ((u & 1) << 1) | ((u & 2) >> 1);
}

// r[j] = 16 bytes (8 bf16: columns 8*dc .. 8*dc+7) of tile row 4u+j, j = 0..3.  Writes the 4x8
// transpose: for each of the 8 columns the 4 consecutive rows as one 8-byte word of the
// transposed tile Xt[column][slot position] (row stride tstr elements); dst = Xt + 8*dc*tstr + 4*pos4(u).
__device__ __forceinline__ void store_transposed_4x8(bf16_t* dst, int tstr, const u32x4* r) {
#pragma unroll
  for (int m = 0; m < 4; ++m) {  // dword m of each row holds columns 2m, 2m+1
    u32x2 lo, hi;
    lo[0] = __builtin_amdgcn_perm(r[1][m], r[0][m], 0x05040100u);
    lo[1] = __builtin_amdgcn_perm(r[3][m], r[2][m], 0x05040100u);
    hi[0] = __builtin_amdgcn_perm(r[1][m], r[0][m], 0x07060302u);
    hi[1] = __builtin_amdgcn_perm(r[3][m], r[2][m], 0x07060302u);
    *reinterpret_cast<u32x2*>(dst + (2 * m) * tstr) = lo;
    *reinterpret_cast<u32x2*>(dst + (2 * m + 1) * tstr) = hi;
  }
}

// LDS exchange inside one wave (a wave's LDS instructions execute in order): only the compiler has to
// be kept from moving the reads above the writes.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The value lane^32 holds, without a trip through LDS: v_permlane32_swap_b32 exchanges the upper 32 lanes
// of its first operand with the lower 32 lanes of its second.  Fed two copies of x it leaves the lower
// half's values in both halves of the first register and the upper half's in both halves of the second.
// Written as an instruction: the compiler's builtin for it returns the first register for both results.
// The no-op covers the wait states the instruction needs after a vector write of its operands.
__device__ __forceinline__ void both_halves(float x, float* lo, float* hi) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  *lo = a;  // x of lane (l & 31)
  *hi = b;  // x of lane (l & 31) + 32
}
__device__ __forceinline__ float max_with_other_half(float x) {
  float lo, hi;
  both_halves(x, &lo, &hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  float lo, hi;
  both_halves(x, &lo, &hi);
  return lo + hi;
}

// XCD-aware work index: every XCD gets one contiguous chunk of the work list, so that neighbours
// in the list (which share K/V or Q/dO rows) meet in the same L2.  Returns -1 for surplus blocks.
__device__ __forceinline__ long xcd_work_index(long total_work) {
  const long chunk = (total_work + NXCD - 1) / NXCD;
  const long local = blockIdx.x / NXCD;
  const long work = (long)(blockIdx.x % NXCD) * chunk + local;
  return (local >= chunk || work >= total_work) ? -1 : work;
}

inline long xcd_grid_blocks(long total_work) { return (total_work + NXCD - 1) / NXCD * NXCD; }

}  // namespace sa
