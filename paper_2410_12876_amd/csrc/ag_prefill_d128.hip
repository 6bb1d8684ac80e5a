// Flag-masked causal prefill attention (Eq. 2 under the mask of Eq. 5), bf16, head dimension 128 -- the
// tuned CDNA4 kernel.  Same formulation as ag_prefill.hip (attention over the compacted rows with the
// per-query boundary cnt[j]; the query's own key/value initialises the online softmax), built for gfx950:
//
//   * K and V tiles (64 cache rows x 256 B) go from global memory straight into LDS with
//     global_load_lds_dwordx4 (no register staging), double-buffered, one workgroup barrier per tile.
//   * Both tiles stay row-major in LDS.  The 16-byte chunk index of a row is XOR-swizzled with a bit-swapped
//     row nibble, applied on the global-address side of the load, so that the 128-bit reads of K fragments
//     (32 consecutive rows, same column) and the transposing reads of V fragments (4 consecutive rows,
//     64 contiguous bytes each) are both free of bank conflicts.
//   * V is never transposed in memory: ds_read_b64_tr_b16 delivers, per lane, four consecutive keys of one
//     head-dim column, which is the A-operand layout of O^T += V^T . P^T.
//   * A lane owns one query: S^T = K . Q^T and O^T = V^T . P^T on v_mfma_f32_32x32x16_bf16, P packed with
//     v_cvt_pk_bf16_f32 straight from the S^T accumulators, row max / sum / rescale as per-lane scalars.
//   * The running maximum is only raised (and O rescaled) when some row's new maximum exceeds it by more than
//     2^8; otherwise the stale maximum is kept, which is exact after the final division by the row sum.
//   * Two workgroups (8 waves) per CU so that one wave's softmax overlaps another's MFMAs; workgroups are
//     numbered so that all tiles of one head land on one XCD (K/V stay in that XCD's L2), longest first.
#include "ag_internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
#define AG_LDS __attribute__((address_space(3)))

constexpr int D = 128;
constexpr int kBN = 64;                   // keys per tile
constexpr int kRowB = D * 2;              // bytes per cache row
constexpr int kTileB = kBN * kRowB;       // 16 KiB per K or V tile
constexpr float kRescaleGap = 8.f;        // log2 units the maximum may lag before O is rescaled

__device__ __forceinline__ int cnt_at(const uint64_t *__restrict__ words, const int32_t *__restrict__ bo, int j) {
  const uint64_t w = words[j >> 6];
  return bo[j >> 6] + __popcll(w & ((1ull << (j & 63)) - 1ull));
}

// swizzle of the 16-byte chunk index of LDS row r: swap the two low bit pairs of r
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  const f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

template <int GB>
__global__ __launch_bounds__(256, 2) void ag_prefill_d128_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint64_t *__restrict__ words, const int32_t *__restrict__ blk_off, const uint16_t *__restrict__ kc,
    const uint16_t *__restrict__ vc, const int64_t *__restrict__ row_off, int L, int Hq, int Hkv, int nw, int n_hy,
    float qscale, uint16_t *__restrict__ out) {
  constexpr int QW = 4 / GB;   // query sub-tiles per workgroup
  constexpr int BM = 32 * QW;  // queries per workgroup
  constexpr int KS = D / 16;   // k-steps of S^T
  constexpr int DT = D / 32;   // 32-row tiles of O^T
  __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * 2 * kTileB];  // [K0][K1][V0][V1], each [row][256 B]

  const int G = Hq / Hkv;
  const int HB = G / GB;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar, so that LDS bases stay in SGPRs
  const int col = lane & 31, hb = lane >> 5;
  // workgroup id -> (query tile, unit/head block): heads vary fastest so that a head keeps its XCD
  const int n_qt = (L + BM - 1) / BM;
  const int hy = blockIdx.x % n_hy;
  const int qtile = n_qt - 1 - blockIdx.x / n_hy;  // longest rows first
  const int u = hy / HB;
  const int hblk = hy - u * HB;
  const int b = u / Hkv, g = u - b * Hkv;
  const int head = g * G + hblk * GB + (wave % GB);
  const int j0 = qtile * BM + (wave / GB) * 32;
  const int jq = min(j0 + col, L - 1);

  const uint64_t *wu = words + (size_t)u * nw;
  const int32_t *bo = blk_off + (size_t)u * (nw + 1);
  const int len_u = (int)min((int64_t)bo[nw], row_off[u + 1] - row_off[u]);
  const int cnt_q = cnt_at(wu, bo, jq);
  const int cnt_wave_lo = cnt_at(wu, bo, min(j0, L - 1));
  const int cnt_wave_hi = j0 < L ? cnt_at(wu, bo, min(j0 + 31, L - 1)) : 0;
  const int cnt_blk = min(cnt_at(wu, bo, min(qtile * BM + BM - 1, L - 1)), len_u);
  const int n_tiles = (cnt_blk + kBN - 1) / kBN;

  const size_t qrow = ((size_t)(b * Hq + head) * L + jq) * D;
  const size_t kvrow = ((size_t)u * L + jq) * D;
  const uint16_t *Kc = kc + (size_t)row_off[u] * D;
  const uint16_t *Vc = vc + (size_t)row_off[u] * D;

  // ---- tile loader: wave w fills rows [16w, 16w+16) of the K and V tiles, 4 rows (1 KiB) per instruction ----
  // lane -> (row r = 16w + 4i + lane/16, physical chunk p = lane%16); it fetches logical chunk p ^ swz(r).
  // Buffer loads with the LDS modifier: the descriptor ends at the unit's last valid row, so rows past the end
  // arrive as zeros (their scores are masked anyway) and nothing outside the unit's slab is ever read.  The
  // loads are issued from inline assembly so that the compiler does not serialise later LDS reads of the
  // *other* buffer behind them; completion is awaited explicitly (s_waitcnt vmcnt(0)) before the barrier that
  // publishes the tile.
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Kc, 0, len_u * kRowB, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Vc, 0, len_u * kRowB, 0x00020000);
  const int ld_r = lane >> 4;
  int ld_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    ld_off[i] = (16 * wave + 4 * i + ld_r) * kRowB + (((lane & 15) ^ ((ld_r << 2) | i)) << 4);  // chunk (lane%16)^swz(r)
  const uint32_t lds_base = (uint32_t)(size_t)((AG_LDS uint8_t *)smem) + wave * 16 * kRowB;
  auto issue_k = [&](int tile) {
    const int soff = tile * kTileB;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t dk = lds_base + (tile & 1) * kTileB + i * 4 * kRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dk), "v"(ld_off[i]), "s"(k_rsrc), "s"(soff) : "memory");
    }
  };
  auto issue_v = [&](int tile) {
    const int soff = tile * kTileB;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t dv = lds_base + 2 * kTileB + (tile & 1) * kTileB + i * 4 * kRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dv), "v"(ld_off[i]), "s"(v_rsrc), "s"(soff) : "memory");
    }
  };
  if (n_tiles > 0) { issue_k(0); issue_v(0); }
  if (n_tiles > 1) issue_k(1);

  // ---- Q fragments (B operand of S^T): lane (query col, half hb), k-step ks: Q[j][16 ks + 8 hb .. +8) ----
  uint4 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const uint4 *>(q + qrow + 16 * ks + 8 * hb);

  // ---- own-token term: initial online-softmax state ----
  float s_self = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const uint4 kr = *reinterpret_cast<const uint4 *>(k + kvrow + 16 * ks + 8 * hb);
    const uint32_t qa[4] = {qf[ks].x, qf[ks].y, qf[ks].z, qf[ks].w}, ka[4] = {kr.x, kr.y, kr.z, kr.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s_self = fmaf(__uint_as_float(qa[e] << 16), __uint_as_float(ka[e] << 16), s_self);
      s_self = fmaf(__uint_as_float(qa[e] & 0xffff0000u), __uint_as_float(ka[e] & 0xffff0000u), s_self);
    }
  }
  s_self += __shfl_xor(s_self, 32, 64);
  float m_run = s_self * qscale;       // reference maximum of the exponentials, log2 units
  float l_run = hb == 0 ? 1.f : 0.f;   // each half of a column holds part of the row sum
  f32x16 acc_o[DT];                    // O^T: acc_o[dt][r] = (d = 32 dt + 8 (r/4) + 4 hb + r%4, query col)
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const uint2 vr = *reinterpret_cast<const uint2 *>(v + kvrow + 32 * dt + 8 * r4 + 4 * hb);
      acc_o[dt][4 * r4 + 0] = __uint_as_float(vr.x << 16);
      acc_o[dt][4 * r4 + 1] = __uint_as_float(vr.x & 0xffff0000u);
      acc_o[dt][4 * r4 + 2] = __uint_as_float(vr.y << 16);
      acc_o[dt][4 * r4 + 3] = __uint_as_float(vr.y & 0xffff0000u);
    }

  // ---- loop-invariant LDS byte offsets of this lane's fragments ----
  // K fragment (A of S^T): row 32 sub + col, logical chunk 2 ks + hb
  int k_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    k_off[ks] = col * kRowB + (((2 * ks + hb) ^ swz(col)) << 4);
    asm volatile("" : "+v"(k_off[ks]));  // keep the offset in a register instead of recomputing the swizzle per tile
  }
  // V fragment (A of O^T) by transposing read: 16-lane group gl = lane/16 covers d = 32 dt + 16 (gl%2) + 0..15 and
  // key half hbv = gl/2; lane i = lane%16 supplies the address of row (4 hbv + i/4 [+ 8]), columns 4 (i%4) .. +3
  const int gl = lane >> 4, li = lane & 15;
  const int v_row = 4 * (gl >> 1) + (li >> 2);
  int v_off[DT][2];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const int r = v_row + 8 * h2;
      const int c = 4 * dt + 2 * (gl & 1) + ((li & 3) >> 1);
      v_off[dt][h2] = r * kRowB + ((c ^ swz(r)) << 4) + (li & 1) * 8;
      asm volatile("" : "+v"(v_off[dt][h2]));
    }

  // ---- software pipeline: S^T of tile t+1 is issued while the softmax of tile t runs ----
  // K runs one tile ahead of V.  At the top of step t (after the barrier) K(t+1) and V(t) are resident; the
  // step then requests K(t+2) into the K buffer that tile t used and V(t+1) into the V buffer of tile t-1.
  auto s_tile = [&](int tile, f32x16 (&acc)[2]) {  // acc = K(tile) . Q^T
    const AG_LDS uint8_t *Kt = (const AG_LDS uint8_t *)smem + (tile & 1) * kTileB;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[sub][r] = 0.f;
    bf16x8 ka[KS][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
        ka[ks][sub] = *reinterpret_cast<const AG_LDS bf16x8 *>(Kt + sub * 32 * kRowB + k_off[ks]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
        acc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks][sub], __builtin_bit_cast(bf16x8, qf[ks]), acc[sub], 0, 0, 0);
  };
  uint4 pf[2][2];  // P fragments (B operand of O^T), [sub][16-key slab]
  float alpha_pending = 1.f;
  bool any_raise = false;
  // softmax of one tile held in acc (key = c0 + 32 sub + 8 (r/4) + 4 hb + r%4, query = col) -> pf, l_run, m_run
  auto softmax_tile = [&](int c0, f32x16 (&acc)[2]) {
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[sub][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * qscale;
    // The reference maximum is raised only when a row exceeds it by more than 2^kRescaleGap; each lane uses
    // its own factor (1 when it has no need), so a query never depends on the queries sharing its wave.
    const bool raise = mx > m_run + kRescaleGap;
    const float m_new = raise ? mx : m_run;
    alpha_pending = __builtin_amdgcn_exp2f(m_run - m_new);
    any_raise = __any(raise);
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(fmaf(acc[sub][r], qscale, -m_run));
        psum += p[r];
      }
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
        pf[sub][sl] = make_uint4(pack2(p[8 * sl + 0], p[8 * sl + 1]), pack2(p[8 * sl + 2], p[8 * sl + 3]),
                                 pack2(p[8 * sl + 4], p[8 * sl + 5]), pack2(p[8 * sl + 6], p[8 * sl + 7]));
    }
    l_run = l_run * alpha_pending + psum;
  };
  auto mask_tile = [&](int c0, f32x16 (&acc)[2]) {
    if (c0 + kBN > cnt_wave_lo) {  // the tile crosses some query's boundary: mask keys >= cnt_q
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = c0 + 32 * sub + 8 * (r >> 2) + 4 * hb + (r & 3);
          if (key >= cnt_q) acc[sub][r] = -INFINITY;
        }
    }
  };
  auto pv_tile = [&](int tile) {  // O^T += V(tile)^T . P^T, after the pending rescale
    if (any_raise) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha_pending;
    }
    const AG_LDS uint8_t *Vt = (const AG_LDS uint8_t *)smem + 2 * kTileB + (tile & 1) * kTileB;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const AG_LDS uint8_t *base = Vt + (32 * sub + 16 * sl) * kRowB;
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(base + v_off[dt][0]));
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(base + v_off[dt][1]));
          const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pf[sub][sl]), acc_o[dt], 0, 0, 0);
        }
    // V fragment reads run four MFMAs ahead of their use
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
      if (i < 12) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
  };
  // one pipeline step: cur holds S^T of tile t; nxt receives S^T of tile t+1
  auto step = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of K(t+1), V(t) has landed
    __syncthreads();                                  // ... and everyone's; step t-1 is fully consumed
    if (t + 2 < n_tiles) issue_k(t + 2);
    if (t + 1 < n_tiles) issue_v(t + 1);
    const int c0 = t * kBN;
    const bool vis_cur = c0 < cnt_wave_hi;                                  // wave-uniform
    const bool vis_nxt = t + 1 < n_tiles && c0 + kBN < cnt_wave_hi;         // wave-uniform
    if (vis_cur) mask_tile(c0, cur);
    if (vis_nxt) {
      s_tile(t + 1, nxt);      // MFMA stream ...
      softmax_tile(c0, cur);   // ... and an independent VALU stream; the groups below interleave them:
      // 4 K-fragment reads ahead, then per MFMA one more read and a slice of the softmax arithmetic
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < 12) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);
      }
    } else if (vis_cur) {
      softmax_tile(c0, cur);
    }
    if (vis_cur) pv_tile(t);
  };
  f32x16 acc_a[2], acc_b[2];
  if (n_tiles > 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (cnt_wave_hi > 0) s_tile(0, acc_a);
  }
  for (int t = 0; t < n_tiles; t += 2) {
    step(t, acc_a, acc_b);
    if (t + 1 < n_tiles) step(t + 1, acc_b, acc_a);
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (j0 + col < L) {
    const float inv = 1.f / l_tot;
    uint16_t *orow = out + qrow;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const uint2 o = make_uint2(pack2(acc_o[dt][4 * r4 + 0] * inv, acc_o[dt][4 * r4 + 1] * inv),
                                   pack2(acc_o[dt][4 * r4 + 2] * inv, acc_o[dt][4 * r4 + 3] * inv));
        *reinterpret_cast<uint2 *>(orow + 32 * dt + 8 * r4 + 4 * hb) = o;
      }
  }
}

}  // namespace

hipError_t ag_launch_prefill_d128(hipStream_t s, const void *q, const void *k, const void *v, const uint64_t *words,
                                  const int32_t *blk_off, int B, int L, int Hq, int Hkv, float qscale, const void *kc,
                                  const void *vc, const int64_t *row_off, void *out) {
  const int nw = ag_nwords(L);
  const int G = Hq / Hkv;
  const int GB = G >= 4 ? 4 : G;
  const int BM = 32 * (4 / GB);
  const int n_hy = B * Hkv * (G / GB);
  const int64_t blocks = (int64_t)((L + BM - 1) / BM) * n_hy;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(256);
#define AG_PF(GG)                                                                                                   \
  hipLaunchKernelGGL((ag_prefill_d128_kernel<GG>), grid, block, 0, s, (const uint16_t *)q, (const uint16_t *)k,        \
                     (const uint16_t *)v, words, blk_off, (const uint16_t *)kc, (const uint16_t *)vc, row_off, L, Hq, \
                     Hkv, nw, n_hy, qscale, (uint16_t *)out)
  if (GB == 1) AG_PF(1); else if (GB == 2) AG_PF(2); else AG_PF(4);
#undef AG_PF
  return hipGetLastError();
}
