// Flag-masked causal prefill attention, bf16, head dimension 128: the 64-queries-per-wave variant of the kernel in
// ag_prefill_d128.hip.  An experiment (selected by AG_PREFILL_Q64=1 in the environment), correct and parity-tested,
// but slower than the 4-wave kernel as the compiler builds it; kept for the measurement it documents.
#include "ag_prefill_bf16_common.h"

namespace {

constexpr int D = 128;
constexpr int kRowB = pf_geom<D>::kRowB, kTileB = pf_geom<D>::kTileB, kGroupB = pf_geom<D>::kGroupB;
__device__ __forceinline__ int swz(int r) { return pf_geom<D>::swz(r); }

// The same attention with 64 queries per wave: two waves per workgroup, each owning TWO 32-query groups (for one
// query head: 64 consecutive queries; for grouped-query attention: the same 32 queries of two heads of the group).
// Every K fragment read from LDS then feeds two S^T MFMAs and every V^T fragment two O^T MFMAs, which halves the
// LDS traffic per MFMA -- the kernel is limited by power, and with it by the energy spent per MFMA.  A wave needs
// about 450 registers for that (two sets of O^T and S^T accumulators and of Q fragments), so one wave runs per SIMD;
// two workgroups of two waves share a CU and the launch has the same shape (128-query items, 2 workgroups per CU)
// as the 4-wave kernel, whose plan, key-chunk split and state layout it shares: "virtual wave" vw = 2 wave + group
// plays the part of that kernel's wave index.  No recent-token variant (that one stays on the 4-wave kernel).
template <int GB>
__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(1, 1))) void ag_prefill_d128_q64_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint64_t *__restrict__ words, const int32_t *__restrict__ blk_off, const uint16_t *__restrict__ kc,
    const uint16_t *__restrict__ vc, const int64_t *__restrict__ row_off, int L, int Hq, int Hkv, int nw, int n_hy,
    int n_split, int n_sp, const int32_t *__restrict__ chunk_tiles_dev, float qscale,
    const int32_t *__restrict__ order, int head_major, uint16_t *__restrict__ out, int out_token_major,
    float *__restrict__ part, int32_t *__restrict__ tickets) {
  constexpr int NW = 2, QG = 2, VW = NW * QG;
  constexpr int QW = VW / GB;    // query sub-tiles per workgroup
  constexpr int RPW = kBN / NW;  // tile rows each wave loads
  constexpr int LI = RPW / 4;    // load instructions per wave and tile (4 rows each)
  constexpr int BM = 32 * QW;    // queries per workgroup
  constexpr int KS = D / 16;
  constexpr int DT = D / 32;
  __shared__ __attribute__((aligned(1024))) uint8_t smem[kGroupB];  // [K0][K1][V0][V1], each [row][256 B]

  const int G = Hq / Hkv;
  const int HB = G / GB;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, hb = lane >> 5;
  const int n_qt = (L + BM - 1) / BM;
  const int per_qt = n_hy * n_split;
  const int split_blocks = n_sp * per_qt;
  int rem, chunk, qt_idx;
  if ((int)blockIdx.x < split_blocks) {
    rem = blockIdx.x % per_qt;
    chunk = rem / n_hy;
    qt_idx = blockIdx.x / per_qt;
  } else {
    const int r2 = blockIdx.x - split_blocks;
    rem = r2 % n_hy;
    chunk = 0;
    qt_idx = n_sp + r2 / n_hy;
  }
  if (head_major) {
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
    rem = (j / n_qt) * 8 + x;
    qt_idx = j % n_qt;
    if (rem >= n_hy) return;
  }
  const int qtile = n_qt - 1 - qt_idx;
  const int pos = rem % n_hy;
  int hy = pos;
  if (order && !head_major) {
    const int n_slot = n_hy >> 3;
    hy = order[(((pos >> 3) + qt_idx) % n_slot) * 8 + (pos & 7)];
  }
  const int u = hy / HB;
  const int hblk = hy - u * HB;
  const int b = u / Hkv, g = u - b * Hkv;

  const uint64_t *wu = words + (size_t)u * nw;
  const int32_t *bo = blk_off + (size_t)u * (nw + 1);
  const int jb = min(qtile * BM + BM - 1, L - 1);
  const uint64_t word_b = wu[jb >> 6];
  const int pre_b = bo[jb >> 6], kept_u = bo[nw];
  const int chunk_tiles = chunk_tiles_dev ? *chunk_tiles_dev : 0x7fffffff / kBN;
  const int64_t ro0 = row_off[u], ro1 = row_off[u + 1];
  const int len_u = (int)min((int64_t)kept_u, ro1 - ro0);
  auto cnt_in = [](uint64_t w, int pre, int j) { return pre + __popcll(w & ((1ull << (j & 63)) - 1ull)); };
  auto in_cache = [&](uint64_t w, int pre, int j) { return ((w >> (j & 63)) & 1ull) != 0 && cnt_in(w, pre, j) < len_u; };
  auto bnd_in = [&](uint64_t w, int pre, int j) { return cnt_in(w, pre, j) + (in_cache(w, pre, j) ? 1 : 0); };
  // per query group of this wave
  int head[QG], j0[QG], jq[QG], pre_w[QG], cnt_q[QG], cnt_lo[QG], cnt_hi[QG];
  uint64_t word_w[QG];
  bool own_kv[QG];
#pragma unroll
  for (int gi = 0; gi < QG; ++gi) {
    const int vw = wave * QG + gi;
    head[gi] = g * G + hblk * GB + (vw % GB);
    j0[gi] = qtile * BM + (vw / GB) * 32;
    jq[gi] = min(j0[gi] + col, L - 1);
    const int jw = min(j0[gi], L - 1) >> 6;
    word_w[gi] = wu[jw];
    pre_w[gi] = bo[jw];
    cnt_q[gi] = min(bnd_in(word_w[gi], pre_w[gi], jq[gi]), len_u);
    own_kv[gi] = chunk == 0 && !in_cache(word_w[gi], pre_w[gi], jq[gi]);
    cnt_lo[gi] = min(bnd_in(word_w[gi], pre_w[gi], min(j0[gi], L - 1)), len_u);
    cnt_hi[gi] = j0[gi] < L ? min(bnd_in(word_w[gi], pre_w[gi], min(j0[gi] + 31, L - 1)), len_u) : 0;
  }
  const int cnt_wave_hi = max(cnt_hi[0], cnt_hi[1]);
  const int cnt_blk = min(bnd_in(word_b, pre_b, jb), len_u);
  const int n_tiles = (cnt_blk + kBN - 1) / kBN;
  const int tile0 = chunk > 0 ? chunk * chunk_tiles : 0;
  if (chunk > 0 && tile0 >= n_tiles) return;
  const int n_chunks = max(1, (n_tiles + chunk_tiles - 1) / chunk_tiles);
  const int n_steps = max(0, min(n_tiles - tile0, chunk_tiles));

  const uint16_t *Kc = kc + (size_t)ro0 * D;
  const uint16_t *Vc = vc + (size_t)ro0 * D;
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Kc, 0, len_u * kRowB, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Vc, 0, len_u * kRowB, 0x00020000);
  const int ld_r = lane >> 4;
  int ld_off[LI];
#pragma unroll
  for (int i = 0; i < LI; ++i) {
    const int r = RPW * wave + 4 * i + ld_r;
    ld_off[i] = r * kRowB + (((lane & 15) ^ swz(r)) << 4);
  }
  const uint32_t ld_base = (uint32_t)(size_t)((AG_LDS uint8_t *)smem) + wave * RPW * kRowB;
  auto issue_k = [&](int i_step) {
    const int soff = (tile0 + i_step) * kTileB;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const uint32_t dk = ld_base + (i_step & 1) * kTileB + i * 4 * kRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dk), "v"(ld_off[i]), "s"(k_rsrc), "s"(soff) : "memory");
    }
  };
  auto issue_v = [&](int i_step) {
    const int soff = (tile0 + i_step) * kTileB;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const uint32_t dv = ld_base + 2 * kTileB + (i_step & 1) * kTileB + i * 4 * kRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dv), "v"(ld_off[i]), "s"(v_rsrc), "s"(soff) : "memory");
    }
  };
  if (n_steps > 0) { issue_k(0); issue_v(0); }
  if (n_steps > 1) issue_k(1);

  // ---- Q fragments and, for chunk 0, each query's own key / value row, one group after the other, through the
  // wave's 8 KiB corner of the V1 buffer (32 rows per pass; see the 4-wave kernel for the layout) ----
  uint4 qf[QG][KS];
  float m_run[QG], l_run[QG];
  f32x16 acc_o[QG][DT];
  {
    const int srow = lane >> 4, schunk = lane & 15;
    AG_LDS uint8_t *stage = (AG_LDS uint8_t *)smem + 3 * kTileB + wave * (kTileB / NW);
    auto wave_sync = [] {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto put = [&](const u32x4 (&x)[8]) {
      wave_sync();
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = 4 * j + srow;
        *reinterpret_cast<AG_LDS u32x4 *>(stage + r * 256 + ((schunk ^ (r & 15)) << 4)) = x[j];
      }
      wave_sync();
    };
    auto get4 = [&](int off) {
      const u32x4 x = *reinterpret_cast<const AG_LDS u32x4 *>(stage + off);
      return make_uint4(x[0], x[1], x[2], x[3]);
    };
    const int rr = col, rk = col & 15;  // this lane's row of the pass and its swizzle key
#pragma unroll
    for (int gi = 0; gi < QG; ++gi) {
      u32x4 sq[8], sk[8], sv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = min(j0[gi] + 4 * j + srow, L - 1);
        const int kv_row = (chunk == 0 && !in_cache(word_w[gi], pre_w[gi], row)) ? row : min(j0[gi], L - 1);
        sq[j] = *reinterpret_cast<const u32x4 *>(q + ((size_t)(b * Hq + head[gi]) * L + row) * D + 8 * schunk);
        sk[j] = *reinterpret_cast<const u32x4 *>(k + ((size_t)u * L + kv_row) * D + 8 * schunk);
        sv[j] = *reinterpret_cast<const u32x4 *>(v + ((size_t)u * L + kv_row) * D + 8 * schunk);
      }
      put(sq);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[gi][ks] = get4(rr * 256 + (((2 * ks + hb) ^ rk) << 4));
      m_run[gi] = kEmptyMax;
      l_run[gi] = 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[gi][dt][r] = 0.f;
      if (chunk == 0) {
        put(sk);
        float s_self = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const uint4 kr = get4(rr * 256 + (((2 * ks + hb) ^ rk) << 4));
          const uint32_t qa[4] = {qf[gi][ks].x, qf[gi][ks].y, qf[gi][ks].z, qf[gi][ks].w};
          const uint32_t ka[4] = {kr.x, kr.y, kr.z, kr.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            s_self = fmaf(__uint_as_float(qa[e] << 16), __uint_as_float(ka[e] << 16), s_self);
            s_self = fmaf(__uint_as_float(qa[e] & 0xffff0000u), __uint_as_float(ka[e] & 0xffff0000u), s_self);
          }
        }
        s_self += __shfl_xor(s_self, 32, 64);
        m_run[gi] = own_kv[gi] ? s_self * qscale : kEmptyMax;
        l_run[gi] = own_kv[gi] && hb == 0 ? 1.f : 0.f;
        put(sv);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const u32x2 x = *reinterpret_cast<const AG_LDS u32x2 *>(stage + rr * 256 + (((4 * dt + r4) ^ rk) << 4) + 8 * hb);
            acc_o[gi][dt][4 * r4 + 0] = own_kv[gi] ? __uint_as_float(x[0] << 16) : 0.f;
            acc_o[gi][dt][4 * r4 + 1] = own_kv[gi] ? __uint_as_float(x[0] & 0xffff0000u) : 0.f;
            acc_o[gi][dt][4 * r4 + 2] = own_kv[gi] ? __uint_as_float(x[1] << 16) : 0.f;
            acc_o[gi][dt][4 * r4 + 3] = own_kv[gi] ? __uint_as_float(x[1] & 0xffff0000u) : 0.f;
          }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the corner is read out before anyone may load V(1) over it
  }
  __builtin_amdgcn_sched_barrier(0);

  int k_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    k_off[ks] = col * kRowB + (((2 * ks + hb) ^ swz(col)) << 4);
    asm volatile("" : "+v"(k_off[ks]));
  }
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

  const AG_LDS uint8_t *lds_grp = (const AG_LDS uint8_t *)smem;
  // The pipeline runs in half tiles of 32 keys (that keeps one S^T accumulator set per group in flight instead of
  // two: 64 registers less).  acc[gi] = K(rows 32 sub .. of the tile of step i_step) . Q_gi^T; every K fragment is
  // read once and used for both groups.
  auto s_half = [&](int i_step, int sub, f32x16 (&acc)[QG]) {
    const AG_LDS uint8_t *Kt = lds_grp + (i_step & 1) * kTileB + sub * 32 * kRowB;
#pragma unroll
    for (int gi = 0; gi < QG; ++gi)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[gi][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 ka = *reinterpret_cast<const AG_LDS bf16x8 *>(Kt + k_off[ks]);
#pragma unroll
      for (int gi = 0; gi < QG; ++gi)
        acc[gi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, __builtin_bit_cast(bf16x8, qf[gi][ks]), acc[gi], 0, 0, 0);
    }
  };
  uint4 pf[QG][2];  // P fragments of the half tile, [group][16-key slab]
  float alpha_pending[QG] = {1.f, 1.f}, psum[QG];
  bool any_raise = false;
  auto weights = [&](f32x16 &acc, int gi) {
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    float ps = 0.f, p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(fmaf(acc[r], qscale, -m_run[gi]));
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
      pf[gi][sl] = make_uint4(pack2(p[8 * sl + 0], p[8 * sl + 1]), pack2(p[8 * sl + 2], p[8 * sl + 3]),
                              pack2(p[8 * sl + 4], p[8 * sl + 5]), pack2(p[8 * sl + 6], p[8 * sl + 7]));
      ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[gi][sl].x), ones, ps, false);
      ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[gi][sl].y), ones, ps, false);
      ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[gi][sl].z), ones, ps, false);
      ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[gi][sl].w), ones, ps, false);
    }
    psum[gi] = ps;
  };
  auto softmax_half = [&](f32x16 (&acc)[QG]) {  // the common case of the 4-wave kernel's softmax, both groups
#pragma unroll
    for (int gi = 0; gi < QG; ++gi) {
      weights(acc[gi], gi);
      alpha_pending[gi] = 1.f;
    }
    any_raise = __any(!(psum[0] <= kLazyLimit) || !(psum[1] <= kLazyLimit));
  };
  auto softmax_raise = [&](f32x16 (&acc)[QG]) {
#pragma unroll
    for (int gi = 0; gi < QG; ++gi) {
      const uint64_t big = __ballot(!(psum[gi] <= kLazyLimit));
      const bool mine = (((big | (big >> 32) | (big << 32)) >> lane) & 1ull) != 0;
      float mx = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[gi][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * qscale;
      const bool up = mine && mx > m_run[gi];
      const float m_new = up ? mx : m_run[gi];
      alpha_pending[gi] = up ? __builtin_amdgcn_exp2f(m_run[gi] - m_new) : 1.f;
      m_run[gi] = m_new;
      weights(acc[gi], gi);
    }
  };
  auto mask_half = [&](int c0, f32x16 (&acc)[QG]) {  // c0 = first key of the half tile
#pragma unroll
    for (int gi = 0; gi < QG; ++gi)
      if (c0 + 32 > cnt_lo[gi]) {  // the half tile crosses some boundary of this group (wave-uniform)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = c0 + 8 * (r >> 2) + 4 * hb + (r & 3);
          if (key >= cnt_q[gi]) acc[gi][r] = -INFINITY;
        }
      }
  };
  auto vis = [&](int i, int sub) -> bool { return (tile0 + i) * kBN + 32 * sub < cnt_wave_hi; };
  // O_gi^T += V(rows 32 sub .. of the tile)^T . P_gi^T: every V^T fragment read once for both groups
  auto pv_half = [&](int i_step, int sub) {
    if (any_raise) {
#pragma unroll
      for (int gi = 0; gi < QG; ++gi)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[gi][dt][r] *= alpha_pending[gi];
    }
    const AG_LDS uint8_t *Vt = lds_grp + 2 * kTileB + (i_step & 1) * kTileB + 32 * sub * kRowB;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const AG_LDS uint8_t *base = Vt + 16 * sl * kRowB;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(base + v_off[dt][0]));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(base + v_off[dt][1]));
        const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int gi = 0; gi < QG; ++gi)
          acc_o[gi][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pf[gi][sl]), acc_o[gi][dt], 0, 0, 0);
      }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 1);
      if (i < 6) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
  };
  // One half tile: cur holds S^T of (step i, half sub); nxt receives the next half's, which is (i, 1) or (i + 1, 0).
  auto half = [&](int i, int sub, f32x16 (&cur)[QG], f32x16 (&nxt)[QG]) {
    const int c0 = (tile0 + i) * kBN + 32 * sub;
    const int ni = sub ? i + 1 : i, nsub = sub ^ 1;
    const bool vis_cur = vis(i, sub);
    const bool vis_nxt = ni < n_steps && vis(ni, nsub);
    if (vis_cur) mask_half(c0, cur);
    if (vis_nxt) {
      s_half(ni, nsub, nxt);
      softmax_half(cur);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        if (n < 6) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);
      }
      if (any_raise) softmax_raise(cur);
    } else if (vis_cur) {
      softmax_half(cur);
      if (any_raise) softmax_raise(cur);
    }
    if (vis_cur) {
#pragma unroll
      for (int gi = 0; gi < QG; ++gi) l_run[gi] = l_run[gi] * alpha_pending[gi] + psum[gi];
      pv_half(i, sub);
    }
  };
  f32x16 acc_a[QG], acc_b[QG];
  if (n_steps > 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (vis(0, 0)) s_half(0, 0, acc_a);
  }
  // Step i = tile i in two halves.  The first half forms S^T of the tile's second half from K(i), the second half
  // that of the next tile's first half from K(i+1); both halves take their values from V(i).  So K(i) is free after
  // the first half and V(i) after the second: K(i+2) is requested at the barrier between the halves and V(i+1) at the
  // barrier on top, each a whole step before its first use.  Loads complete in order, so waiting until at most the
  // LI loads of the younger request are outstanding (vmcnt(LI)) is waiting for the older one.
  static_assert(LI == 8, "the s_waitcnt immediates below are LI");
  for (int i = 0; i < n_steps; ++i) {
    if (i >= 1 && i + 1 < n_steps) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");  // V(i); K(i+1) may be in flight
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();            // V(i) is there for everyone; everyone is done with V(i-1)
    if (i + 1 < n_steps) issue_v(i + 1);
    half(i, 0, acc_a, acc_b);
    if (i + 1 < n_steps) {
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");  // K(i+1); V(i+1) may be in flight
      __syncthreads();          // K(i+1) is there for everyone; everyone is done with K(i)
      if (i + 2 < n_steps) issue_k(i + 2);
    }
    half(i, 1, acc_b, acc_a);
  }

  // ---- an item cut into chunks: as in the 4-wave kernel, the state of virtual wave vw at [item][chunk][vw] ----
  bool writer = true;
  if (n_chunks > 1) {
    const size_t item = (size_t)qtile * n_hy + hy;
    const size_t cstride = (size_t)VW * 66 * 64;
#pragma unroll
    for (int gi = 0; gi < QG; ++gi) {
      float *mine = part + ((item * n_split + chunk) * VW + wave * QG + gi) * (66 * 64) + lane;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          __hip_atomic_store(&mine[(16 * dt + r) * 64], acc_o[gi][dt][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(&mine[64 * 64], m_run[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(&mine[65 * 64], l_run[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int *last = reinterpret_cast<int *>(smem);
    if (tid == 0)
      *last = __hip_atomic_fetch_add(&tickets[item], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_chunks - 1;
    __syncthreads();
    writer = *last != 0;
    if (writer) {
      auto peek = [](const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); };
#pragma unroll
      for (int gi = 0; gi < QG; ++gi) {
        const float *st = part + ((item * n_split) * VW + wave * QG + gi) * (66 * 64) + lane;
        float m = m_run[gi];
        for (int c = 0; c < n_chunks; ++c)
          if (c != chunk) m = fmaxf(m, peek(&st[c * cstride + 64 * 64]));
        if (n_chunks == 2) {
          const float f_own = __builtin_amdgcn_exp2f(m_run[gi] - m);
          l_run[gi] = mul_round(l_run[gi], f_own);
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[gi][dt][r] = mul_round(acc_o[gi][dt][r], f_own);
        } else {
          l_run[gi] = 0.f;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[gi][dt][r] = 0.f;
        }
        for (int c = 0; c < n_chunks; ++c) {
          if (n_chunks == 2 && c == chunk) continue;
          const float *sc = st + c * cstride;
          const float f = __builtin_amdgcn_exp2f(peek(&sc[64 * 64]) - m);
          l_run[gi] = mul_round_add(peek(&sc[65 * 64]), f, l_run[gi]);
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              acc_o[gi][dt][r] = mul_round_add(peek(&sc[(16 * dt + r) * 64]), f, acc_o[gi][dt][r]);
        }
      }
    }
  }
  if (!writer) return;
  __syncthreads();  // every wave is done with the K/V tiles
#pragma unroll
  for (int gi = 0; gi < QG; ++gi) {
    const float l_tot = l_run[gi] + __shfl_xor(l_run[gi], 32, 64);
    const float inv = 1.f / l_tot;
    AG_LDS uint8_t *ost = (AG_LDS uint8_t *)smem + (wave * QG + gi) * (32 * kRowB);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const u32x2 o = {pack2(acc_o[gi][dt][4 * r4 + 0] * inv, acc_o[gi][dt][4 * r4 + 1] * inv),
                         pack2(acc_o[gi][dt][4 * r4 + 2] * inv, acc_o[gi][dt][4 * r4 + 3] * inv)};
        *reinterpret_cast<AG_LDS u32x2 *>(ost + col * kRowB + (((4 * dt + r4) ^ (col & 15)) << 4) + 8 * hb) = o;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int row_stride = (out_token_major ? Hq : 1) * kRowB;
    uint16_t *obase = out + (out_token_major ? (((size_t)b * L + j0[gi]) * Hq + head[gi]) * D
                                             : ((size_t)(b * Hq + head[gi]) * L + j0[gi]) * D);
    const int n_rows = min(32, L - j0[gi]);
    const __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)obase, 0, n_rows > 0 ? (uint32_t)((n_rows - 1) * row_stride + kRowB) : 0u, 0x00020000);
    const int orow_l = lane >> 4, ochunk = lane & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 4 * i + orow_l;
      const u32x4 x = *reinterpret_cast<const AG_LDS u32x4 *>(ost + row * kRowB + ((ochunk ^ (row & 15)) << 4));
      if (row < n_rows) __builtin_amdgcn_raw_buffer_store_b128(x, o_rsrc, orow_l * row_stride + ochunk * 16, i * 4 * row_stride, 0);
    }
  }
}

}  // namespace

hipError_t ag_launch_prefill_d128_q64(hipStream_t s, const void *q, const void *k, const void *v, const uint64_t *words,
                                      const int32_t *blk_off, int L, int Hq, int Hkv, float qscale, const void *kc,
                                      const void *vc, const int64_t *row_off, void *out, const ag_pf_plan &plan,
                                      float *part, bool out_token_major, ag_evpair ev, unsigned blocks) {
  const int nw = ag_nwords(L);
  const int G = Hq / Hkv;
  const int GB = G >= 4 ? 4 : G;
  const dim3 grid(blocks), block(128);
#define AG_PQ(GG)                                                                                                   \
  AG_LAUNCH(ev, (ag_prefill_d128_q64_kernel<GG>), grid, block, 0, s, (const uint16_t *)q, (const uint16_t *)k,       \
            (const uint16_t *)v, words, blk_off, (const uint16_t *)kc, (const uint16_t *)vc, row_off, L, Hq, Hkv, nw, \
            plan.n_hy, plan.n_split, plan.n_sp, plan.chunk_tiles, qscale, plan.order, plan.head_major, (uint16_t *)out, \
            out_token_major ? 1 : 0, part, plan.tickets)
  if (GB == 1) { AG_PQ(1); } else if (GB == 2) { AG_PQ(2); } else { AG_PQ(4); }
#undef AG_PQ
  return hipGetLastError();
}
