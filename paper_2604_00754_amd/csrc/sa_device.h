// Small device-side helpers used by every kernel file of libsa (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sa {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// two bf16 packed in one dword -> two floats
__device__ __forceinline__ float bf16lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// round-to-nearest-even float -> bf16 pair packed in a dword (lo = a, hi = b)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float sigmoidf_exact(float x) { return 1.0f / (1.0f + __expf(-x)); }
// The same with the hardware reciprocal (1 ulp) in place of the IEEE division sequence (a dozen instructions):
// for results that are rounded to bf16 anyway.  Exact at both infinities (1 / inf = 0, 1 / 1 = 1).
__device__ __forceinline__ float sigmoidf_rcp(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// Original index of the token at slot `slot` (identity when perm is null).
__device__ __forceinline__ int slot_to_orig(const int32_t* __restrict__ perm, int slot) {
  return perm ? perm[slot] : slot;
}

// Reduce an unwrapped slot t in (-n, 2n) to 0..n-1.
__device__ __forceinline__ int wrap_slot(int t, int n) {
  t = t < 0 ? t + n : t;
  return t >= n ? t - n : t;
}

__device__ __forceinline__ float load_gate(const void* g, size_t idx, int f32) {
  if (f32) return reinterpret_cast<const float*>(g)[idx];
  return bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(g)[idx]);
}

__device__ __forceinline__ void store_gate(void* g, size_t idx, int f32, float v) {
  if (f32) {
    reinterpret_cast<float*>(g)[idx] = v;
  } else {
    reinterpret_cast<uint16_t*>(g)[idx] = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
  }
}

}  // namespace sa
