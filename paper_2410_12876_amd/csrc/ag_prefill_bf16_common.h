// Shared by the bf16 prefill kernels (ag_prefill_bf16.hip: 4 waves x 32 queries, head dimension 128 or 64, the one in
// use; ag_prefill_d128_q64.hip: 2 waves x 64 queries, head dimension 128, an experiment): tile geometry, the LDS
// swizzle, packing and the never-contracted multiply-adds of the chunk merge.
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

constexpr int kBN = 64;                    // keys per tile
constexpr float kLazyLimit = 1073741824.f; // 2^30: a lane's sum of weights above this raises its reference maximum
constexpr float kEmptyMax = -1.0e30f;      // "no key seen yet" reference maximum (finite on purpose)

// Tile geometry for head dimension HD (128 or 64): a K or V tile is 64 rows of HD bf16, row-major in LDS, its
// 16-byte chunks XOR-swizzled with a key taken from the row so that the three access patterns -- 1 KiB contiguous
// from the loads, 32 rows x one chunk for the K fragments, 4 rows x 64 contiguous bytes for the transposing V
// reads -- are all free of bank conflicts.
//   HD = 128: a row covers all 64 banks; key = the row's nibble with its two bit pairs swapped.
//   HD = 64:  a row covers half of the banks (even rows one half, odd rows the other).  With t = (row / 2) % 8 the
//             key is (t % 2) * 4 + t / 2: the eight rows of equal parity among 16 consecutive ones get eight different
//             keys (K fragments), and rows r, r + 2 move a quad of chunks to the other quad (V reads).
template <int HD>
struct pf_geom {
  static constexpr int kRowB = HD * 2;          // bytes per row
  static constexpr int kTileB = kBN * kRowB;    // bytes per K or V tile
  static constexpr int kGroupB = 4 * kTileB;    // LDS per workgroup: [K0][K1][V0][V1]
  static constexpr int CPR = kRowB / 16;        // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;          // rows one 64-lane load or store instruction covers
  static constexpr int kState = (HD / 2 + 2) * 64;  // floats of one wave's partial state: O^T, then m, then l
  static __device__ __forceinline__ int swz(int r) {
    if (HD == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
    const int t = (r >> 1) & 7;
    return ((t & 1) << 2) | (t >> 1);
  }
  // key of the per-wave staging areas (query rows in, output rows out)
  static __device__ __forceinline__ int key(int r) { return HD == 128 ? (r & 15) : ((r >> 1) & 7); }
};

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
