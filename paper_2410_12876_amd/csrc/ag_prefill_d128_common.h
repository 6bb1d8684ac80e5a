// Shared by the two bf16, D = 128 prefill kernels (ag_prefill_d128.hip: 4 waves x 32 queries, the one in use;
// ag_prefill_d128_q64.hip: 2 waves x 64 queries, an experiment): tile geometry, the LDS swizzle, packing and the
// never-contracted multiply-adds of the chunk merge.
#pragma once
#include "ag_internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
#define AG_LDS __attribute__((address_space(3)))

constexpr int D = 128;
constexpr int kBN = 64;                   // keys per tile
constexpr int kRowB = D * 2;              // bytes per cache row
constexpr int kTileB = kBN * kRowB;       // 16 KiB per K or V tile
constexpr int kGroupB = 4 * kTileB;       // LDS per group: [K0][K1][V0][V1]
constexpr float kLazyLimit = 1073741824.f; // 2^30: a lane's sum of weights above this raises its reference maximum
constexpr float kEmptyMax = -1.0e30f;     // "no key seen yet" reference maximum (finite on purpose)

// swizzle of the 16-byte chunk index of LDS row r: swap the two low bit pairs of r
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  const f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// a * b rounded, then + c rounded: never contracted into a fused multiply-add (whose result would depend on which
// of two chunk states plays the part of c), whatever the compiler's contraction setting
__device__ __forceinline__ float mul_round_add(float a, float b, float c) {
#pragma clang fp contract(off)
  const float prod = a * b;
  return prod + c;
}
__device__ __forceinline__ float mul_round(float a, float b) {
#pragma clang fp contract(off)
  return a * b;
}

}  // namespace
