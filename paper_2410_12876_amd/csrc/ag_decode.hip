// Decode attention over ragged per-(batch, KV head) caches (Sec. 3.1, decoding stage) -- split-K.
//
// The step is bandwidth-bound: every cached K and V row is read once.  Work is cut into items of kChunk rows
// of one unit; the item list is built on the device from len[] (no host read-back), and a persistent grid
// walks it round-robin.  Inside an item each group of LPR lanes owns one row per load (16 bytes per lane, a
// wave reads 1 KiB of contiguous rows per instruction), keeps an online-softmax state per query head of the
// group, and the states are merged through LDS into one (max, sum, weighted-V) record per item and head.
// A second kernel merges the records of each (batch, query head) with the new token's own key/value -- the
// diagonal of Eq. 5 -- normalises, and appends the new row to the cache when its flag says so.
#include <mutex>

#include "ag_internal.h"

// Scratch of ag_decode_attn_static, the entry point for callers that cannot allocate: the per-item records the
// two decode kernels exchange live here instead of in a context's workspace.  One copy per GPU, held until the
// process ends.  In host code this name is only a stand-in for the symbol; the device address comes from
// hipGetSymbolAddress (ag_static_scratch below) and is what every launch receives.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kChunk = 128;      // rows per work item
constexpr int kWgsPerCu = 2;     // persistent workgroups per CU (measured on 1024 ragged caches: 2 -> 5.7 TB/s,
                                 // 3 -> 5.3, 4 -> 5.4, 1 -> 4.6; fewer concurrent streams keep DRAM pages open)
constexpr int kMaxUnits = 8192;  // units whose item offsets fit in LDS
constexpr float kLog2e = 1.4426950408889634f;

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t nt_u32x4;

template <typename T> struct elems;  // element count, widening and dot product of one 16-byte vector
template <> struct elems<float> {
  static constexpr int n = 4;
  static __device__ __forceinline__ void widen(const uint4 &r, float *f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  static __device__ __forceinline__ float dot(const uint4 &a, const uint4 &b) {
    float d = __uint_as_float(a.x) * __uint_as_float(b.x);
    d = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), d);
    d = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), d);
    return fmaf(__uint_as_float(a.w), __uint_as_float(b.w), d);
  }
};
template <> struct elems<uint16_t> {  // bf16 bit patterns
  static constexpr int n = 8;
  static __device__ __forceinline__ void widen(const uint4 &r, float *f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  // 8 bf16 products summed in fp32 by v_dot2c_f32_bf16, two per instruction, without widening either operand
  static __device__ __forceinline__ float dot(const uint4 &a, const uint4 &b) {
    float d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.x), __builtin_bit_cast(bf16x2, b.x), 0.f, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.y), __builtin_bit_cast(bf16x2, b.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.z), __builtin_bit_cast(bf16x2, b.z), d, false);
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.w), __builtin_bit_cast(bf16x2, b.w), d, false);
  }
};

__device__ __forceinline__ float widen1(float x) { return x; }
__device__ __forceinline__ float widen1(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ __forceinline__ void narrow1(float x, float *o) { *o = x; }
__device__ __forceinline__ void narrow1(float x, uint16_t *o) {  // round to nearest even
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  *o = (uint16_t)(u >> 16);
}

// valid rows of a unit, never more than its slab holds
__device__ __forceinline__ int unit_len(const int32_t *__restrict__ len, const int64_t *__restrict__ row_off, int u) {
  const int64_t cap = row_off[u + 1] - row_off[u];
  const int n = len[u];
  return n < 0 ? 0 : (n < cap ? n : (int)cap);
}

template <int CTRL> __device__ __forceinline__ float dpp(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
// Sum over aligned groups of LPR lanes; every lane of the group gets the sum.
template <int LPR> __device__ __forceinline__ float group_sum(float x) {
  x += dpp<0xB1>(x);                           // quad_perm [1,0,3,2]
  x += dpp<0x4E>(x);                           // quad_perm [2,3,0,1]
  if (LPR >= 8) x += dpp<0x141>(x);            // row_half_mirror
  if (LPR >= 16) x += dpp<0x140>(x);           // row_mirror
  if (LPR >= 32) x += __shfl_xor(x, 16, 64);
  if (LPR >= 64) x += __shfl_xor(x, 32, 64);
  return x;
}

// ---------------------------------------------------------------------------------------------------------
// Kernel 1: per-item partial attention.
//   item_off [U+1] (global copy for the merge kernel), pm/pl [items*G], pacc [items*G, D]
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void ag_decode_partial_kernel(const T *__restrict__ q, const T *__restrict__ kc,
                                                                const T *__restrict__ vc,
                                                                const int64_t *__restrict__ row_off,
                                                                const int32_t *__restrict__ len, int U, int Hkv,
                                                                int meta_lds, int grid_stream, float qscale,
                                                                int32_t *__restrict__ item_off_g,
                                                                float *__restrict__ pm, float *__restrict__ pl,
                                                                float *__restrict__ pacc) {
  constexpr int EPL = elems<T>::n;        // elements per lane
  constexpr int LPR = D / EPL;            // lanes per row
  constexpr int GPW = 64 / LPR;           // rows per wave load
  constexpr int NST = 4 * GPW;            // online-softmax states per block
  constexpr int NIT = kChunk / 4 / GPW;   // loads that cover a wave's quarter of an item
  constexpr int UN = (G <= 2 ? 8 : 4) < NIT ? (G <= 2 ? 8 : 4) : NIT;  // rows in flight per lane group
  static_assert(NIT % UN == 0, "a wave's rows must be a whole number of batches");
  extern __shared__ int32_t smem[];
  int32_t *item_off = smem;               // [U+1]
  int32_t *scan = smem + (U + 1);         // [256]
  float *st = reinterpret_cast<float *>(scan + 256);  // [NST][G][D+2]
  // with few enough units their lengths and slab offsets also live in LDS, so that starting an item costs no
  // round trip to memory
  int32_t *s_len = reinterpret_cast<int32_t *>(st + (size_t)NST * G * (D + 2));  // [U]     (meta_lds)
  int64_t *s_ro = reinterpret_cast<int64_t *>((reinterpret_cast<uintptr_t>(s_len + U) + 7) & ~uintptr_t(7));  // [U]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // ---- item offsets: exclusive scan of ceil(len/kChunk) over units ----
  const int per = (U + 255) / 256;
  const int u0 = tid * per, u1 = min(U, u0 + per);
  int32_t sum = 0;
  for (int u = u0; u < u1; ++u) {
    const int n_u = unit_len(len, row_off, u);
    if (meta_lds) { s_len[u] = n_u; s_ro[u] = row_off[u]; }
    sum += (n_u + kChunk - 1) / kChunk;
  }
  // exclusive scan over the 256 threads: inside a wave by shuffles, across the four waves through LDS (one barrier)
  int32_t incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) scan[wave] = incl;
  __syncthreads();
  int32_t run = incl - sum;
  for (int w = 0; w < wave; ++w) run += scan[w];
  for (int u = u0; u < u1; ++u) {
    item_off[u] = run;
    run += (unit_len(len, row_off, u) + kChunk - 1) / kChunk;
  }
  if (tid == 255) item_off[U] = scan[0] + scan[1] + scan[2] + scan[3];
  __syncthreads();
  const int n_items = item_off[U];
  if (blockIdx.x == 0)
    for (int u = tid; u <= U; u += 256) item_off_g[u] = item_off[u];

  const int grp = lane / LPR, seg = lane % LPR;
  // The launch holds more workgroups than the streaming regime wants (grid_stream = kWgsPerCu per CU).  If every
  // item can have a workgroup of its own, it gets one -- a small step is one round of loads instead of two; else
  // only the first grid_stream workgroups walk the list.
  const int n_wg = n_items <= (int)gridDim.x ? n_items : min((int)gridDim.x, grid_stream);
  if ((int)blockIdx.x >= n_wg) return;
  for (int item = blockIdx.x; item < n_items; item += n_wg) {
    // unit of this item: last u with item_off[u] <= item
    int lo = 0, hi = U;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (item_off[mid] <= item) lo = mid; else hi = mid;
    }
    const int u = lo;
    const int c = item - item_off[u];
    const int b = u / Hkv, g = u - b * Hkv;
    const int n = meta_lds ? s_len[u] : unit_len(len, row_off, u);
    const int64_t ro = meta_lds ? s_ro[u] : row_off[u];
    const int row_end = min(n, (c + 1) * kChunk);
    const int wrow0 = c * kChunk + wave * (kChunk / 4);
    const uint4 *K = reinterpret_cast<const uint4 *>(kc + (size_t)ro * D);
    const uint4 *V = reinterpret_cast<const uint4 *>(vc + (size_t)ro * D);

    uint4 qr[G];  // this lane's 16 bytes of each query row, as stored; the score is scaled after the sum
#pragma unroll
    for (int gg = 0; gg < G; ++gg) qr[gg] = reinterpret_cast<const uint4 *>(q + ((size_t)(b * Hkv + g) * G + gg) * D)[seg];
    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) {
      m[gg] = -INFINITY; l[gg] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[gg][e] = 0.f;
    }

    for (int it0 = 0; it0 < NIT; it0 += UN) {
      if (wrow0 + it0 * GPW >= row_end) break;  // wave-uniform
      uint4 kk[UN], vv[UN];
      bool ok[UN];
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        const int r = wrow0 + (it0 + j) * GPW + grp;
        ok[j] = r < row_end;
        kk[j] = make_uint4(0, 0, 0, 0);
        vv[j] = make_uint4(0, 0, 0, 0);
        if (ok[j]) {  // every cached row is read exactly once per step: non-temporal, so that the stream does not
                      // push the small hot data (queries, lengths, item records) out of the caches (measured on 1024
                      // ragged caches: 200.7 -> 190.4 us per step, and the merge kernel 8.5 -> 6.5 us)
          const nt_u32x4 kx = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4 *>(&K[(size_t)r * LPR + seg]));
          const nt_u32x4 vx = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4 *>(&V[(size_t)r * LPR + seg]));
          kk[j] = make_uint4(kx[0], kx[1], kx[2], kx[3]);
          vv[j] = make_uint4(vx[0], vx[1], vx[2], vx[3]);
        }
      }
      float s[G][UN];
#pragma unroll
      for (int j = 0; j < UN; ++j) {
#pragma unroll
        for (int gg = 0; gg < G; ++gg) {
          const float d = group_sum<LPR>(elems<T>::dot(qr[gg], kk[j])) * qscale;
          s[gg][j] = ok[j] ? d : -INFINITY;
        }
      }
#pragma unroll
      for (int gg = 0; gg < G; ++gg) {
        float mn = m[gg];
#pragma unroll
        for (int j = 0; j < UN; ++j) mn = fmaxf(mn, s[gg][j]);
        if (mn == -INFINITY) continue;  // this lane group has seen no valid row yet
        const float alpha = exp2f(m[gg] - mn);  // m = -inf -> 0
        m[gg] = mn;
        l[gg] *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[gg][e] *= alpha;
#pragma unroll
        for (int j = 0; j < UN; ++j) s[gg][j] = exp2f(s[gg][j] - mn);  // -inf -> 0
      }
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        float vf[EPL];
        elems<T>::widen(vv[j], vf);
#pragma unroll
        for (int gg = 0; gg < G; ++gg) {
          const float p = m[gg] == -INFINITY ? 0.f : s[gg][j];
          l[gg] += p;
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[gg][e] = fmaf(p, vf[e], acc[gg][e]);
        }
      }
    }

    // ---- merge the NST states of the block ----
    const int sidx = wave * GPW + grp;
#pragma unroll
    for (int gg = 0; gg < G; ++gg) {
      float *rec = st + ((size_t)sidx * G + gg) * (D + 2);
      if (seg == 0) { rec[0] = m[gg]; rec[1] = l[gg]; }
#pragma unroll
      for (int e = 0; e < EPL; ++e) rec[2 + seg * EPL + e] = acc[gg][e];
    }
    __syncthreads();
    for (int o = tid; o < G * D; o += 256) {
      const int gg = o / D, d = o - gg * D;
      float M = -INFINITY;
#pragma unroll
      for (int sI = 0; sI < NST; ++sI) M = fmaxf(M, st[((size_t)sI * G + gg) * (D + 2)]);
      float L = 0.f, A = 0.f;
#pragma unroll
      for (int sI = 0; sI < NST; ++sI) {
        const float *rec = st + ((size_t)sI * G + gg) * (D + 2);
        const float w = rec[0] == -INFINITY ? 0.f : exp2f(rec[0] - M);
        L = fmaf(w, rec[1], L);
        A = fmaf(w, rec[2 + d], A);
      }
      const size_t pr = (size_t)item * G + gg;
      pacc[pr * D + d] = A;
      if (d == 0) { pm[pr] = M; pl[pr] = L; }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------------------
// Kernel 2: one block per (batch, query head): merge item records + the new token itself, write out, append.
template <typename T, int D>
__global__ __launch_bounds__(D) void ag_decode_merge_kernel(const T *__restrict__ q, const T *__restrict__ k_new,
                                                            const T *__restrict__ v_new,
                                                            const uint8_t *__restrict__ new_flags, int pos, int Hq,
                                                            int Hkv, float qscale,
                                                            const int32_t *__restrict__ item_off,
                                                            const float *__restrict__ pm, const float *__restrict__ pl,
                                                            const float *__restrict__ pacc, T *__restrict__ kc,
                                                            T *__restrict__ vc, int32_t *__restrict__ idx,
                                                            const int64_t *__restrict__ row_off,
                                                            int32_t *__restrict__ len, T *__restrict__ out,
                                                            int32_t *__restrict__ d_err, ag_ring_dev ring) {
  __shared__ float red[D / 64 > 0 ? D / 64 : 1];
  __shared__ float wts[64];
  const int G = Hq / Hkv;
  const int bi = blockIdx.x;  // b * Hq + i
  const int b = bi / Hq, i = bi - b * Hq;
  const int g = i / G, gg = i - g * G;
  const int u = b * Hkv + g;
  const int d = threadIdx.x, lane = d & 63;
  // Everything that does not depend on another load is requested here, in one round trip: the launch is short and
  // latency-bound, so the number of dependent round trips is its cost.
  const T kn_raw = k_new[(size_t)u * D + d], vn_raw = v_new[(size_t)u * D + d];
  const float kn = widen1(kn_raw), vn = widen1(vn_raw);
  const float qd = widen1(q[(size_t)bi * D + d]) * qscale;
  const int i0 = item_off[u], i1 = item_off[u + 1];
  const bool keep_new = new_flags == nullptr || new_flags[u] != 0;
  const int n_len = len[u];
  const int64_t r0 = row_off[u], cap = row_off[u + 1] - r0;

  // A batch of up to 64 item records: lane j takes the maximum and sum of record base + j; every thread also
  // requests its column of the batch's first 8 records, so that they travel together with the maxima.
  auto request = [&](int base, float &mj, float &lj, float (&x)[8]) {
    const int n = min(64, i1 - base);
    const size_t pr = (size_t)(base + lane) * G + gg;
    mj = lane < n ? pm[pr] : -INFINITY;
    lj = lane < n ? pl[pr] : 0.f;
    const float *col = pacc + ((size_t)base * G + gg) * D + d;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = e < n ? col[(size_t)e * G * D] : 0.f;
  };
  float mj = -INFINITY, lj = 0.f, x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (i0 < i1) request(i0, mj, lj, x);

  // self score: scale * q . k_new (in log2 units)
  float part = qd * kn;
  for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
  if ((d & 63) == 0) red[d >> 6] = part;
  __syncthreads();
  float s_self = 0.f;
#pragma unroll
  for (int w = 0; w < (D + 63) / 64; ++w) s_self += red[w];

  float M = s_self, L = 1.f, A = vn;  // state so far: the new token alone, relative to M
  // recent-token ring (Table 6 of the appendix): an evicted token among the n_recent - 1 positions before `pos` is still visible
  // (the kept ones are cache rows already).  Slot contents are block-uniform, so the branches are too.
  if (ring.k) {
    const T *rk = static_cast<const T *>(ring.k), *rv = static_cast<const T *>(ring.v);
    for (int w = 0; w < ring.n; ++w) {
      const size_t slot = (size_t)u * ring.n + w;
      const int p = ring.pos[slot];
      if (!(p < pos && p > pos - ring.n) || ring.flags[slot] != 0) continue;
      float part_r = qd * widen1(rk[slot * D + d]);
      for (int o = 32; o > 0; o >>= 1) part_r += __shfl_xor(part_r, o, 64);
      __syncthreads();  // red[] of the previous reduction is consumed
      if ((d & 63) == 0) red[d >> 6] = part_r;
      __syncthreads();
      float sr = 0.f;
#pragma unroll
      for (int xw = 0; xw < (D + 63) / 64; ++xw) sr += red[xw];
      const float M_new = fmaxf(M, sr);
      const float keep = exp2f(M - M_new), pr = exp2f(sr - M_new);
      M = M_new;
      L = L * keep + pr;
      A = fmaf(pr, widen1(rv[slot * D + d]), A * keep);
    }
  }
  // the wave reduces the batch's maximum and sum, the weights go through LDS, and every thread then adds its
  // column with independent loads
  for (int base = i0; base < i1; base += 64) {
    const int n = min(64, i1 - base);
    if (base != i0) request(base, mj, lj, x);
    float mb = mj;
    for (int o = 32; o > 0; o >>= 1) mb = fmaxf(mb, __shfl_xor(mb, o, 64));
    const float M_new = fmaxf(M, mb);
    const float keep = exp2f(M - M_new);
    const float wj = lane < n ? exp2f(mj - M_new) : 0.f;
    float lsum = wj * lj;
    for (int o = 32; o > 0; o >>= 1) lsum += __shfl_xor(lsum, o, 64);
    __syncthreads();  // wts of the previous batch are consumed
    if (d < 64) wts[d] = wj;
    __syncthreads();
    M = M_new;
    L = L * keep + lsum;
    A *= keep;
    const float *col = pacc + ((size_t)base * G + gg) * D + d;
#pragma unroll
    for (int e = 0; e < 8; ++e) A = fmaf(e < n ? wts[e] : 0.f, x[e], A);
    int j = 8;
    for (; j + 8 <= n; j += 8) {
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] = col[(size_t)(j + e) * G * D];
#pragma unroll
      for (int e = 0; e < 8; ++e) A = fmaf(wts[j + e], y[e], A);
    }
    for (; j < n; ++j) A = fmaf(wts[j], col[(size_t)j * G * D], A);
  }
  narrow1(A / L, &out[(size_t)bi * D + d]);

  if (gg == 0 && keep_new) {
    __syncthreads();  // every thread has read len[u] before it changes
    if (n_len < cap) {
      kc[(size_t)(r0 + n_len) * D + d] = kn_raw;
      vc[(size_t)(r0 + n_len) * D + d] = vn_raw;
      if (d == 0) { idx[r0 + n_len] = pos; len[u] = n_len + 1; }
    } else if (d == 0) {
      atomicOr(d_err, 1);
    }
  }
  // The new token takes the ring slot pos % n_recent.  That slot held position pos - n_recent, which no query
  // head of this step can see any more, and a reader that races with the write skips the slot whether it finds
  // the old position (out of the window) or the new one (not before pos).
  if (ring.k && gg == 0) {
    const size_t slot = (size_t)u * ring.n + (size_t)(pos % ring.n);
    static_cast<T *>(ring.k)[slot * D + d] = kn_raw;
    static_cast<T *>(ring.v)[slot * D + d] = vn_raw;
    if (d == 0) {
      ring.flags[slot] = keep_new ? 1 : 0;
      ring.pos[slot] = pos;
    }
  }
}

// After prefilling: the ring takes the last min(L, n_recent) prompt tokens of every unit (kept or not); the other
// slots are marked empty.  One workgroup per unit, one wave per token slot in turn.
template <typename T>
__global__ __launch_bounds__(256) void ag_ring_fill_kernel(const T *__restrict__ k, const T *__restrict__ v,
                                                           const uint8_t *__restrict__ flags, int L, int D, int pos0,
                                                           ag_ring_dev ring) {
  const int u = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int w = wave; w < ring.n; w += 4) {
    // slot w holds the position p with p % n == w among the last n positions before pos0 + L, if it is a prompt token
    const int end = pos0 + L;                                   // first position after the prompt
    const int p = end - 1 - ((end - 1 - w) % ring.n + ring.n) % ring.n;  // largest p < end with p % n == w
    const int t = p - pos0;
    const size_t slot = (size_t)u * ring.n + w;
    if (t >= 0 && t < L && p >= 0) {
      for (int d = lane; d < D; d += 64) {
        static_cast<T *>(ring.k)[slot * D + d] = k[((size_t)u * L + t) * D + d];
        static_cast<T *>(ring.v)[slot * D + d] = v[((size_t)u * L + t) * D + d];
      }
      if (lane == 0) { ring.flags[slot] = flags[(size_t)u * L + t] != 0; ring.pos[slot] = p; }
    } else if (lane == 0) {
      ring.flags[slot] = 1;
      ring.pos[slot] = kRingEmpty;
    }
  }
}

int64_t max_items(int units, int64_t cache_rows) { return cache_rows / kChunk + units; }

template <typename T, int D, int G>
hipError_t launch_t(ag_ctx *ctx, hipStream_t s, const void *q, const void *k_new, const void *v_new,
                    const uint8_t *new_flags, int pos, int B, int Hq, int Hkv, float scale, void *kc, void *vc,
                    int32_t *idx, const int64_t *row_off, int32_t *len, int64_t total_rows, void *out, ws_cursor &ws,
                    ag_ring_dev ring) {
  const int num_cu = ctx->num_cu;
  int32_t *d_err = ctx->d_err;
  const int U = B * Hkv;
  const int64_t items = max_items(U, total_rows);
  int32_t *item_off = ws.take<int32_t>(U + 1);
  float *pm = ws.take<float>(items * G);
  float *pl = ws.take<float>(items * G);
  float *pacc = ws.take<float>(items * G * D);
  if (!ws.ok) return hipSuccess;
  constexpr int EPL = elems<T>::n, LPR = D / EPL, GPW = 64 / LPR, NST = 4 * GPW;
  const int meta_lds = U <= 2048;
  const size_t shmem = (size_t)(U + 1 + 256) * 4 + (size_t)NST * G * (D + 2) * 4 +
                       (meta_lds ? (size_t)U * 4 + 8 + (size_t)U * 8 : 0);
  const float qscale = scale * kLog2e;
  const int grid_stream = num_cu * kWgsPerCu;
  int blocks = 2 * grid_stream;  // the kernel uses them all only when that gives every item its own workgroup
  if (blocks > items) blocks = (int)items;
  if (blocks < 1) blocks = 1;
  if (shmem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ag_decode_partial_kernel<T, D, G>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
  }
  AG_LAUNCH(ag_time_kernel(ctx, AG_K_DECODE_PARTIAL), (ag_decode_partial_kernel<T, D, G>), dim3(blocks), dim3(256), shmem, s, (const T *)q,
                     (const T *)kc, (const T *)vc, row_off, len, U, Hkv, meta_lds, grid_stream, qscale, item_off, pm, pl, pacc);
  AG_LAUNCH(ag_time_kernel(ctx, AG_K_DECODE_MERGE), (ag_decode_merge_kernel<T, D>), dim3(B * Hq), dim3(D), 0, s, (const T *)q, (const T *)k_new,
                     (const T *)v_new, new_flags, pos, Hq, Hkv, qscale, item_off, pm, pl, pacc, (T *)kc, (T *)vc, idx,
                     row_off, len, (T *)out, d_err, ring);
  return hipGetLastError();
}

template <typename T, int D, typename... A>
hipError_t launch_g(int G, A &&...a) {
  switch (G) {
    case 1: return launch_t<T, D, 1>(a...);
    case 2: return launch_t<T, D, 2>(a...);
    case 4: return launch_t<T, D, 4>(a...);
    case 8: return launch_t<T, D, 8>(a...);
  }
  return hipErrorInvalidValue;
}

}  // namespace

size_t ag_ws_decode_bytes(int units, int G, int D, int64_t cache_rows) {
  const int64_t items = max_items(units, cache_rows);
  return ag_align256((size_t)(units + 1) * 4) + 2 * ag_align256((size_t)items * G * 4) +
         ag_align256((size_t)items * G * D * 4);
}

// Device address of this GPU's copy of `scratch`, looked up once per device (with that device current) and kept.
hipError_t ag_static_scratch(int device, char **ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static char *known[kMaxDevices];
  *ptr = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!known[device]) {
    hipError_t e = hipSetDevice(device);
    if (e != hipSuccess) return e;
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    known[device] = static_cast<char *>(p);
  }
  *ptr = known[device];
  return hipSuccess;
}

bool ag_decode_supported(ag_dtype dt, int D, int G, int units) {
  if (units > kMaxUnits) return false;
  if (!(G == 1 || G == 2 || G == 4 || G == 8)) return false;
  return dt == AG_BF16 ? (D == 64 || D == 128) : (D == 64 || D == 128);
}

hipError_t ag_launch_decode(ag_ctx *ctx, hipStream_t s, const void *q, const void *k_new, const void *v_new,
                            const uint8_t *new_flags, int pos, int B, int Hq, int Hkv, int D, ag_dtype dt,
                            float scale, void *kc, void *vc, int32_t *idx, const int64_t *row_off, int32_t *len,
                            int64_t total_rows, void *out, ws_cursor &ws, ag_ring_dev ring) {
  const int G = Hq / Hkv;
#define AG_DEC(T, DD)                                                                                              \
  return launch_g<T, DD>(G, ctx, s, q, k_new, v_new, new_flags, pos, B, Hq, Hkv, scale, kc, vc, idx, row_off, len, \
                         total_rows, out, ws, ring)
  if (dt == AG_BF16) {
    if (D == 64) AG_DEC(uint16_t, 64);
    if (D == 128) AG_DEC(uint16_t, 128);
  } else {
    if (D == 64) AG_DEC(float, 64);
    if (D == 128) AG_DEC(float, 128);
  }
#undef AG_DEC
  return hipErrorInvalidValue;
}

hipError_t ag_launch_ring_fill(hipStream_t s, const void *k, const void *v, const uint8_t *flags, int units, int L,
                               int D, ag_dtype dt, int pos0, ag_ring_dev ring) {
  if (dt == AG_BF16)
    hipLaunchKernelGGL(ag_ring_fill_kernel<uint16_t>, dim3(units), dim3(256), 0, s, (const uint16_t *)k,
                       (const uint16_t *)v, flags, L, D, pos0, ring);
  else
    hipLaunchKernelGGL(ag_ring_fill_kernel<float>, dim3(units), dim3(256), 0, s, (const float *)k, (const float *)v,
                       flags, L, D, pos0, ring);
  return hipGetLastError();
}
