// Flag-masked causal prefill attention (Eq. 2 under the mask of Eq. 5), over COMPACTED keys: dispatch, and the fp32
// kernel.
//
// Because the cache keeps surviving rows in token order, the keys visible to query j are exactly the first
// cnt[j] cache rows of its KV head (cnt = exclusive prefix count of the flags) plus the query's own k_j, v_j.
// So the kernels are causal flash attention over a shorter key sequence with the per-query boundary cnt[j], and
// the own-token term is folded in as the initial state of the online softmax (which also keeps every running
// maximum finite).  The work is (1 - evicted fraction) of dense causal attention for any flag pattern; tiles
// that hold only evicted keys do not exist.  bf16 (head dimension 128 or 64) runs on the MFMA kernel of
// ag_prefill_bf16.hip; fp32 on the plain-ALU kernel below (config 1 is a correctness configuration).
#include "ag_internal.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// exclusive prefix count of the keep flags at token j of one unit
__device__ __forceinline__ int cnt_at(const uint64_t *__restrict__ words, const int32_t *__restrict__ bo, int j) {
  const uint64_t w = words[j >> 6];
  return bo[j >> 6] + __popcll(w & ((1ull << (j & 63)) - 1ull));
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
  const float qscale = scale * kLog2e;
  if (dt == AG_BF16)
    return ag_launch_prefill_bf16(s, q, k, v, words, blk_off, B, L, Hq, Hkv, D, qscale, n_recent, kc, vc, row_off, out,
                                  plan, part, false, ag_time_kernel(ctx, AG_K_PREFILL));
  ag_tick(ctx, AG_K_PREFILL, s);
  {
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
