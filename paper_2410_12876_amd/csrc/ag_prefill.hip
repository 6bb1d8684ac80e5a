// Flag-masked causal prefill attention (Eq. 2 under the mask of Eq. 5), over COMPACTED keys.
//
// Because the cache keeps surviving rows in token order, the keys visible to query j are exactly the first
// cnt[j] cache rows of its KV head (cnt = exclusive prefix count of the flags) plus the query's own k_j, v_j.
// So the kernel is causal flash attention over a shorter key sequence with the per-query boundary cnt[j], and
// the own-token term is folded in as the initial state of the online softmax (which also keeps every running
// maximum finite).  The work is (1 - evicted fraction) of dense causal attention for any flag pattern; tiles
// that hold only evicted keys do not exist.
//
// bf16 path, one workgroup = 4 waves; a wave owns 32 queries of one head.  Everything is laid out so that a
// lane owns one query (column) of each MFMA tile:
//   S^T[key, query] = K_tile . Q^T        v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers)
//   O^T[d,   query] += V_tile^T . P^T     A = V^T from LDS, B = P straight from the S^T accumulators
// Row maximum, sum and rescale are then per-lane scalars (one cross-lane exchange between lane and lane^32).
#include "ag_internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kBN = 64;  // keys per tile

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {  // round to nearest even
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7fffu + ((a >> 16) & 1u);
  b += 0x7fffu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xffff0000u);
}

// exclusive prefix count of the keep flags at token j of one unit
__device__ __forceinline__ int cnt_at(const uint64_t *__restrict__ words, const int32_t *__restrict__ bo, int j) {
  const uint64_t w = words[j >> 6];
  return bo[j >> 6] + __popcll(w & ((1ull << (j & 63)) - 1ull));
}

// Keep bits of mask word t of a unit restricted to the tokens that are among the unit's len_u compacted rows: all
// kept ones, unless the cache overflowed -- a kept token that found no room is not there, and the recent-token band
// must show it like an evicted one.
__device__ __forceinline__ uint64_t in_cache_bits(const uint64_t *__restrict__ words, const int32_t *__restrict__ bo,
                                                  int t, int len_u) {
  uint64_t w = words[t];
  const int room = len_u - bo[t];
  if (room <= 0) return 0;
  while (__popcll(w) > room) w &= ~(1ull << (63 - __clzll(w)));  // (never entered without an overflow)
  return w;
}

// GB = query heads of one KV group handled by a workgroup (one per wave); 4/GB query sub-tiles of 32.
template <int D, int GB>
__global__ __launch_bounds__(256) void ag_prefill_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint64_t *__restrict__ words, const int32_t *__restrict__ blk_off, const uint16_t *__restrict__ kc,
    const uint16_t *__restrict__ vc, const int64_t *__restrict__ row_off, int L, int Hq, int Hkv, int nw,
    float qscale, int n_recent, uint16_t *__restrict__ out) {
  constexpr int QW = 4 / GB;       // query sub-tiles per workgroup
  constexpr int BM = 32 * QW;      // queries per workgroup
  constexpr int KS = D / 16;       // MFMA k-steps over the head dimension
  constexpr int DT = D / 32;       // 32-row tiles of O^T
  constexpr int KSTR = D + 8;      // LDS row stride of the K tile (bf16 elements)
  constexpr int VSTR = kBN + 8;    // LDS row stride of the V^T tile
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * KSTR];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[D * VSTR];
  __shared__ uint32_t nf_rows[3][2];  // per band tile: rows whose value row held a NaN or an infinity (see `tile`)

  const int G = Hq / Hkv;
  const int HB = G / GB;  // head blocks per KV group
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, hb = lane >> 5;
  const int qtile = gridDim.x - 1 - blockIdx.x;  // longest rows first
  const int u = blockIdx.y / HB;                 // unit = b * Hkv + g
  const int hblk = blockIdx.y - u * HB;
  const int b = u / Hkv, g = u - b * Hkv;
  const int head = g * G + hblk * GB + (wave % GB);
  const int j0 = qtile * BM + (wave / GB) * 32;
  const int jq = min(j0 + col, L - 1);  // this lane's query (clamped; clamped lanes never store)

  const uint64_t *wu = words + (size_t)u * nw;
  const int32_t *bo = blk_off + (size_t)u * (nw + 1);
  // kept rows, clamped to the unit's slab so that an overflowed cache can never be read out of bounds
  const int len_u = (int)min((int64_t)bo[nw], row_off[u + 1] - row_off[u]);
  // (boundaries clamped to the rows the cache holds: after a capacity overflow the rows that did not fit are not
  // there -- their tokens count as evicted -- and the zero rows a tile is padded with are never attended)
  const int cnt_q = min(cnt_at(wu, bo, jq), len_u);
  const int cnt_wave_lo = min(cnt_at(wu, bo, min(j0, L - 1)), len_u);
  const int cnt_wave_hi = j0 < L ? min(cnt_at(wu, bo, min(j0 + 31, L - 1)), len_u) : 0;
  const int cnt_blk = min(cnt_at(wu, bo, min(qtile * BM + BM - 1, L - 1)), len_u);
  if (tid < 6) nf_rows[tid >> 1][tid & 1] = 0u;  // ordered before their first use by the barriers of `tile`
  bool poisoned = false;

  const size_t qrow = ((size_t)(b * Hq + head) * L + jq) * D;
  const size_t kvrow = ((size_t)u * L + jq) * D;

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
  float m_run = s_self * qscale;   // running maximum, log2 units
  float l_run = hb == 0 ? 1.f : 0.f;  // the two halves of a column each hold part of the sum
  f32x16 acc_o[DT];                 // O^T: acc_o[dt][r] = (d = 32 dt + 8 (r/4) + 4 hb + r%4, query col)
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

  const uint16_t *Kc = kc + (size_t)row_off[u] * D;
  const uint16_t *Vc = vc + (size_t)row_off[u] * D;

  // One 64-key tile: rows [r0, r0 + 64) of src_k / src_v (rows outside [0, r_end) read as zero).  Compacted tiles
  // (band == false) hide keys at or past the query's boundary cnt_q.  Band tiles (band == true) come from the
  // uncompacted K/V and show only the evicted tokens (keep bit clear in bword) among the n_recent - 1 tokens just
  // before the query: the kept ones are already among the compacted rows (Table 6 of the appendix, recent-token settings).
  // In a band tile a weight of exactly 0 still meets the masked row's values in O^T += V^T . P^T, and 0 x NaN is
  // NaN: a value row with a NaN or an infinity in it is therefore staged as zeros and noted in nf_rows[bi]; a query
  // that does see such a row gets NaN as its whole output row, and no other query is touched by it.
  auto tile = [&](const uint16_t *src_k, const uint16_t *src_v, int r0, int r_end, bool band, uint64_t bword, int bi) {
    __syncthreads();  // previous tile fully consumed
    // ---- stage K tile (row-major) and V tile (transposed) in LDS ----
    constexpr int CPR = D / 8;  // 16-byte chunks per row
    for (int ch = tid; ch < kBN * CPR; ch += 256) {
      const int r = ch / CPR, sg = ch - r * CPR;
      uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if (r0 + r < r_end) {
        kk = *reinterpret_cast<const uint4 *>(src_k + (size_t)(r0 + r) * D + sg * 8);
        vv = *reinterpret_cast<const uint4 *>(src_v + (size_t)(r0 + r) * D + sg * 8);
      }
      if (band) {  // (workgroup-uniform branch; the CPR lanes of a row are neighbours inside one wave)
        const uint32_t vw[4] = {vv.x, vv.y, vv.z, vv.w};
        bool bad = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) bad |= (vw[e] & 0x7f80u) == 0x7f80u || (vw[e] & 0x7f800000u) == 0x7f800000u;
        const uint64_t row_lanes = ((1ull << CPR) - 1ull) << ((lane / CPR) * CPR);
        if (__ballot(bad) & row_lanes) {
          vv = make_uint4(0, 0, 0, 0);
          if (sg == 0) atomicOr(&nf_rows[bi][r >> 5], 1u << (r & 31));
        }
      }
      *reinterpret_cast<uint4 *>(&Ks[r * KSTR + sg * 8]) = kk;
      const uint32_t va[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        Vt[(sg * 8 + 2 * e) * VSTR + r] = (uint16_t)(va[e] & 0xffffu);
        Vt[(sg * 8 + 2 * e + 1) * VSTR + r] = (uint16_t)(va[e] >> 16);
      }
    }
    __syncthreads();
    // nothing visible to this wave in the tile (wave-uniform)?
    if (band ? (j0 >= L || r0 > j0 + 30 || r0 + kBN - 1 < j0 - (n_recent - 1)) : (r0 >= cnt_wave_hi)) return;

    // ---- S^T = K_tile . Q^T ----
    f32x16 acc_s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_s[sub][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 a = *reinterpret_cast<const uint4 *>(&Ks[(32 * sub + col) * KSTR + 16 * ks + 8 * hb]);
        acc_s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                             __builtin_bit_cast(bf16x8, qf[ks]), acc_s[sub], 0, 0, 0);
      }
    }
    // acc_s[sub][r]: key = r0 + 32 sub + 8 (r/4) + 4 hb + r%4, query = col
    if (band) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const uint32_t wsub = (uint32_t)(bword >> (32 * sub + 4 * hb));  // keep bits of this lane's 16 keys
        const int dl = jq - 1 - r0 - 32 * sub - 4 * hb;                  // (query - 1) - key for c = 0
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 8 * (r >> 2) + (r & 3);
          const bool in_window = (unsigned)(dl - c) < (unsigned)(n_recent - 1);  // query - n_recent < key < query
          if (!in_window || ((wsub >> c) & 1u)) acc_s[sub][r] = -INFINITY;
        }
      }
      // does this query see, through its window, a row that was scrubbed?
      const int lo = max(0, jq - (n_recent - 1) - r0), hi = min(kBN - 1, jq - 1 - r0);
      if (hi >= lo) {
        const uint64_t win = (hi - lo == 63 ? ~0ull : ((1ull << (hi - lo + 1)) - 1ull)) << lo;
        const uint64_t nf = ((uint64_t)nf_rows[bi][1] << 32) | nf_rows[bi][0];
        poisoned |= (win & ~bword & nf) != 0ull;
      }
    } else if (r0 + kBN > cnt_wave_lo) {  // tile crosses some query's boundary: mask keys >= cnt_q
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = r0 + 32 * sub + 8 * (r >> 2) + 4 * hb + (r & 3);
          if (key >= cnt_q) acc_s[sub][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[sub][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * qscale);  // m_run is finite, so m_new is
    const float alpha = exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    uint4 pf[2][2];  // P fragments (B operand of O^T), [sub][16-key slab]
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = exp2f(fmaf(acc_s[sub][r], qscale, -m_new));
        psum += p[r];
      }
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
        pf[sub][sl] = make_uint4(pack_bf16(p[8 * sl + 0], p[8 * sl + 1]), pack_bf16(p[8 * sl + 2], p[8 * sl + 3]),
                                 pack_bf16(p[8 * sl + 4], p[8 * sl + 5]), pack_bf16(p[8 * sl + 6], p[8 * sl + 7]));
    }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha;

    // ---- O^T += V^T . P^T ; A lane (d = 32 dt + col, half hb) needs keys slab + {4hb..4hb+3, 8+4hb..8+4hb+3} ----
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const uint16_t *vp = &Vt[(32 * dt + col) * VSTR + 32 * sub + 16 * sl + 4 * hb];
          const uint2 lo = *reinterpret_cast<const uint2 *>(vp);
          const uint2 hi = *reinterpret_cast<const uint2 *>(vp + 8);
          const uint4 a = make_uint4(lo.x, lo.y, hi.x, hi.y);
          acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                              __builtin_bit_cast(bf16x8, pf[sub][sl]), acc_o[dt], 0, 0, 0);
        }
  };
  for (int c0 = 0; c0 < cnt_blk; c0 += kBN) tile(Kc, Vc, c0, len_u, false, 0, 0);
  if (n_recent > 1) {  // workgroup-uniform: band tiles that can hold a key of one of the workgroup's queries
    const int jb = min(qtile * BM + BM - 1, L - 1);
    const int klo = max(0, qtile * BM - (n_recent - 1)), khi = jb - 1;
    for (int bt = klo >> 6; bt <= (khi >> 6) && khi >= klo; ++bt)  // at most 3 tiles: n_recent <= 64, BM <= 128
      tile(k + (size_t)u * L * D, v + (size_t)u * L * D, bt * kBN, L, true, in_cache_bits(wu, bo, bt, len_u), bt - (klo >> 6));
  }
  if (poisoned) l_run = __builtin_nanf("");

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (j0 + col < L) {
    const float inv = 1.f / l_tot;
    uint16_t *orow = out + qrow;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const uint2 o = make_uint2(pack_bf16(acc_o[dt][4 * r4 + 0] * inv, acc_o[dt][4 * r4 + 1] * inv),
                                   pack_bf16(acc_o[dt][4 * r4 + 2] * inv, acc_o[dt][4 * r4 + 3] * inv));
        *reinterpret_cast<uint2 *>(orow + 32 * dt + 8 * r4 + 4 * hb) = o;
      }
  }
}

// fp32 path (plain ALUs): one wave per (query, head); lanes take keys for the scores and output columns for
// the weighted sum.  A correctness path for small fp32 problems, not a roofline one.
template <int D>
__global__ __launch_bounds__(256) void ag_prefill_f32_kernel(const float *__restrict__ q, const float *__restrict__ k,
                                                             const float *__restrict__ v,
                                                             const uint64_t *__restrict__ words,
                                                             const int32_t *__restrict__ blk_off,
                                                             const float *__restrict__ kc, const float *__restrict__ vc,
                                                             const int64_t *__restrict__ row_off, int L, int Hq,
                                                             int Hkv, int nw, float qscale, int n_recent,
                                                             float *__restrict__ out) {
  constexpr int DPL = (D + 63) / 64;  // output columns per lane
  __shared__ float qs[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 4 + wave;
  const int bh = blockIdx.y;  // b * Hq + head
  const int b = bh / Hq, head = bh - b * Hq;
  const int G = Hq / Hkv;
  const int u = b * Hkv + head / G;
  if (j >= L) return;  // whole wave; no block barrier below
  const float *qr = q + ((size_t)bh * L + j) * D;
  for (int d = lane; d < D; d += 64) qs[wave][d] = qr[d] * qscale;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int64_t cap_u = row_off[u + 1] - row_off[u];  // kept tokens beyond it found no room in the cache
  const int cnt = (int)min((int64_t)cnt_at(words + (size_t)u * nw, blk_off + (size_t)u * (nw + 1), j), cap_u);
  const float *Kc = kc + (size_t)row_off[u] * D;
  const float *Vc = vc + (size_t)row_off[u] * D;
  const float *kself = k + ((size_t)u * L + j) * D;
  const float *vself = v + ((size_t)u * L + j) * D;

  float s_self = 0.f;
  for (int d = 0; d < D; ++d) s_self = fmaf(qs[wave][d], kself[d], s_self);
  float m = s_self, l = 1.f, o[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) o[e] = lane + 64 * e < D ? vself[lane + 64 * e] : 0.f;

  // recent-token band (Table 6 of the appendix): evicted tokens among the n_recent - 1 just before the query stay visible; the
  // kept ones are among the cache rows already.  Wave-uniform loop, one key at a time.
  for (int i = 1; i < n_recent && j - i >= 0; ++i) {
    const int t = j - i;
    if (((words[(size_t)u * nw + (t >> 6)] >> (t & 63)) & 1ull) &&
        cnt_at(words + (size_t)u * nw, blk_off + (size_t)u * (nw + 1), t) < cap_u)
      continue;  // a cache row already
    const float *kr = k + ((size_t)u * L + t) * D, *vr = v + ((size_t)u * L + t) * D;
    float s = 0.f;
    for (int d = 0; d < D; ++d) s = fmaf(qs[wave][d], kr[d], s);
    const float mn = fmaxf(m, s);
    const float alpha = exp2f(m - mn), p = exp2f(s - mn);
    m = mn;
    l = l * alpha + p;
#pragma unroll
    for (int e = 0; e < DPL; ++e)
      if (lane + 64 * e < D) o[e] = fmaf(p, vr[lane + 64 * e], o[e] * alpha);
  }

  for (int c0 = 0; c0 < cnt; c0 += 64) {
    const int c = c0 + lane;
    float s = -INFINITY;
    if (c < cnt) {
      const float *kr = Kc + (size_t)c * D;
      s = 0.f;
      for (int d = 0; d < D; ++d) s = fmaf(qs[wave][d], kr[d], s);
    }
    float mx = s;
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    const float mn = fmaxf(m, mx);
    const float alpha = exp2f(m - mn);
    m = mn;
    const float p = exp2f(s - mn);  // -inf -> 0
    float ps = p;
    for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 64);
    l = l * alpha + ps;
#pragma unroll
    for (int e = 0; e < DPL; ++e) o[e] *= alpha;
    const int nk = min(64, cnt - c0);
    for (int t = 0; t < nk; ++t) {
      const float pt = __shfl(p, t, 64);
      const float *vr = Vc + (size_t)(c0 + t) * D;
#pragma unroll
      for (int e = 0; e < DPL; ++e)
        if (lane + 64 * e < D) o[e] = fmaf(pt, vr[lane + 64 * e], o[e]);
    }
  }
  float *orow = out + ((size_t)bh * L + j) * D;
#pragma unroll
  for (int e = 0; e < DPL; ++e)
    if (lane + 64 * e < D) orow[lane + 64 * e] = o[e] / l;
}

}  // namespace

bool ag_prefill_supported(ag_dtype dt, int D, int G) {
  if (!(G == 1 || G == 2 || G == 4 || G == 8)) return false;
  return dt == AG_BF16 ? (D == 64 || D == 128) : (D == 32 || D == 64 || D == 128 || D == 256);
}

hipError_t ag_launch_prefill(ag_ctx *ctx, hipStream_t s, const void *q, const void *k, const void *v,
                             const uint64_t *words, const int32_t *blk_off, int B, int L, int Hq, int Hkv, int D,
                             ag_dtype dt, float scale, int n_recent, const void *kc, const void *vc,
                             const int64_t *row_off, void *out, const ag_pf_plan &plan, float *part) {
  const int nw = ag_nwords(L);
  const int G = Hq / Hkv;
  const float qscale = scale * kLog2e;
  if (dt == AG_BF16 && D == 128)
    return ag_launch_prefill_d128(s, q, k, v, words, blk_off, B, L, Hq, Hkv, qscale, n_recent, kc, vc, row_off, out, plan,
                                  part, false, ag_time_kernel(ctx, AG_K_PREFILL));
  ag_tick(ctx, AG_K_PREFILL, s);
  if (dt == AG_BF16) {
    const int GB = G >= 4 ? 4 : G;
    const int BM = 32 * (4 / GB);
    const dim3 grid((L + BM - 1) / BM, B * Hkv * (G / GB)), block(256);
#define AG_PF(DD, GG)                                                                                             \
  hipLaunchKernelGGL((ag_prefill_mfma_kernel<DD, GG>), grid, block, 0, s, (const uint16_t *)q, (const uint16_t *)k, \
                     (const uint16_t *)v, words, blk_off, (const uint16_t *)kc, (const uint16_t *)vc, row_off, L, Hq, \
                     Hkv, nw, qscale, n_recent, (uint16_t *)out)
    if (GB == 1) AG_PF(64, 1); else if (GB == 2) AG_PF(64, 2); else AG_PF(64, 4);  // D = 128 took the tuned kernel
#undef AG_PF
  } else {
    const dim3 grid((L + 3) / 4, B * Hq), block(256);
#define AG_PF32(DD)                                                                                              \
  hipLaunchKernelGGL((ag_prefill_f32_kernel<DD>), grid, block, 0, s, (const float *)q, (const float *)k,           \
                     (const float *)v, words, blk_off, (const float *)kc, (const float *)vc, row_off, L, Hq, Hkv, nw, \
                     qscale, n_recent, (float *)out)
    if (D == 32) AG_PF32(32); else if (D == 64) AG_PF32(64); else if (D == 128) AG_PF32(128); else AG_PF32(256);
#undef AG_PF32
  }
  ag_tock(ctx, AG_K_PREFILL, s);
  return hipGetLastError();
}
