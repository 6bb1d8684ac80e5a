// Flag scan and KV stream compaction (Sec. 3.3: k, v of a token stay in the cache iff its flag is 1).
//
// ag_flag_scan turns the byte flags of one (batch, KV head) unit into 64-bit keep masks (one wave64 ballot per
// 64 tokens) and an exclusive prefix count per mask word, 1024 tokens per workgroup; it is what the prefill kernel
// needs when the compacted rows already exist.  ag_scan_compact does the same and the copy in one launch: every
// wave owns one mask word, a lane's rank inside the word plus the word's prefix is the destination row.
#include <string.h>

#include "ag_internal.h"

namespace {

constexpr int kScanThreads = 256;

constexpr int kSegWords = 16;  // mask words (1024 tokens) per scan workgroup

// What the scan leaves for the D = 128 prefill kernel, run by every workgroup of a grid = (segments, units) launch
// after it knows its unit's running total (unit_total is valid in thread 0 of a unit's last segment):
// all workgroups clear the per-item arrival counters; the last segments publish their unit's kept-row count and the
// one that arrives last turns the counts into the plan.  The counts cross workgroups inside one launch, so they
// are written through and read past the caches (system-scope relaxed accesses, complete before the arrival is
// counted) instead of paying for cache-wide fences.
__device__ __forceinline__ void plan_tail(const ag_pf_plan &plan, int num_units, int L, int u, bool last_seg,
                                          int32_t unit_total, int32_t *__restrict__ arrivals) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ int32_t part[kScanThreads / 64];
  if (plan.tickets) {
    const int nb = gridDim.x * gridDim.y, bid = blockIdx.y * gridDim.x + blockIdx.x;
    for (int i = bid * kScanThreads + tid; i < plan.n_items; i += nb * kScanThreads) plan.tickets[i] = 0;
  }
  if (!plan.order && !plan.chunk_tiles) return;
  if (!last_seg) return;  // a unit's last segment knows its total
  __shared__ int is_last;
  if (tid == 0) {
    __hip_atomic_store(&plan.kept[u], unit_total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    is_last = __hip_atomic_fetch_add(arrivals, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.y - 1;
    if (is_last) __hip_atomic_store(arrivals, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
  }
  __syncthreads();
  if (!is_last) return;
  __shared__ int32_t kept[1024];
  for (int i = tid; i < num_units && i < 1024; i += kScanThreads)
    kept[i] = __hip_atomic_load(&plan.kept[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  __syncthreads();
  if (plan.order) {
    // Head blocks are ranked by the kept rows of their unit and dealt to the 8 XCDs in snake order
    // (0..7, 7..0, ...): order[p] is the head block at position p of a row, and position p runs on XCD p % 8.
    __shared__ int32_t kept_h[256];  // kept rows per head block (at most 256 are ordered)
    for (int hy = tid; hy < plan.n_hy && hy < 256; hy += kScanThreads) kept_h[hy] = kept[hy / plan.HB];
    __syncthreads();
    for (int hy = tid; hy < plan.n_hy && hy < 256; hy += kScanThreads) {
      const int mine = kept_h[hy];
      int rank = 0;
      for (int o = 0; o < plan.n_hy; ++o) {
        const int other = kept_h[o];
        rank += (other > mine) || (other == mine && o < hy);
      }
      const int round = rank >> 3, pos = rank & 7;
      plan.order[round * 8 + ((round & 1) ? 7 - pos : pos)] = hy;
    }
  }
  if (plan.chunk_tiles) {
    // Key tiles of all items together (a unit's kept rows taken as evenly spread over its tokens), per
    // workgroup slot of the chip: an item is cut only where it alone would exceed that average, and never
    // into more than n_split chunks.
    const int n_qt = (L + plan.BM - 1) / plan.BM;
    int steps = 0;
    for (int idx = tid; idx < num_units * n_qt; idx += kScanThreads) {
      const int uu = idx / n_qt, t = idx - uu * n_qt;
      const int64_t pos = min((t + 1) * plan.BM, L);
      steps += (int)(((int64_t)kept[uu] * pos / L + 63) / 64);
    }
    for (int o = 32; o > 0; o >>= 1) steps += __shfl_xor(steps, o, 64);
    __syncthreads();
    if (lane == 0) part[wave] = steps;
    __syncthreads();
    if (tid == 0) {
      const int64_t total = (int64_t)(part[0] + part[1] + part[2] + part[3]) * plan.HB;
      // (15 % above the plain average: a model of the launch -- 7 us per workgroup plus 1.7 us per tile on 64 slots
      // per XCD -- and the measurement agree that slightly longer chunks, i.e. fewer cut items, finish earlier)
      int ct = (int)((total * 23 / 20 + plan.slots - 1) / plan.slots);
      const int lo = (plan.max_tiles + plan.n_split - 1) / plan.n_split;
      ct = ct < lo ? lo : ct;
      ct = ct < 8 ? 8 : ct;
      *plan.chunk_tiles = ct;
    }
  }
}


// grid = (segments, units).  A workgroup builds the mask words of its 1024 tokens and needs the number of
// kept tokens before them; it counts those itself (4 flags per load), so no workgroup waits for another.
// flags == nullptr stands for "every token kept" (the attention inside the gate module evicts nothing): the words
// and counts are then written without reading anything.
__global__ __launch_bounds__(kScanThreads) void ag_flag_scan_kernel(const uint8_t *__restrict__ flags, int L, int nw,
                                                                    uint64_t *__restrict__ words,
                                                                    int32_t *__restrict__ blk_off, ag_pf_plan plan,
                                                                    int num_units, int32_t *__restrict__ arrivals) {
  __shared__ int32_t cnts[kSegWords];
  __shared__ int32_t part[kScanThreads / 64];
  const int u = blockIdx.y, seg = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint8_t *f = flags ? flags + (size_t)u * L : nullptr;
  const int w_first = seg * kSegWords;
  const bool last_seg = seg == (int)gridDim.x - 1;

  // this segment's flags first (the loads are independent of the count below)
  constexpr int WPW = kSegWords / (kScanThreads / 64);  // words per wave
  uint8_t fb[WPW];
#pragma unroll
  for (int j = 0; j < WPW; ++j) {
    const int w = w_first + wave * WPW + j;
    const int t = w * 64 + lane;
    fb[j] = (w < nw && t < L) ? (flags ? f[t] : (uint8_t)1) : (uint8_t)0;
  }
  // kept tokens before the segment
  const int t_end = w_first * 64;  // <= L, a multiple of 1024
  int before = 0;
  if (!flags) {
    before = tid == 0 ? t_end : 0;
  } else if ((reinterpret_cast<uintptr_t>(f) & 3) == 0) {
    const uint32_t *f4 = reinterpret_cast<const uint32_t *>(f);
    for (int i = tid; i < t_end / 4; i += kScanThreads) {
      const uint32_t x = f4[i];
      before += __popc((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u);  // non-zero bytes of x
    }
  } else {
    for (int i = tid; i < t_end; i += kScanThreads) before += f[i] != 0;
  }
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o, 64);
  if (lane == 0) part[wave] = before;
#pragma unroll
  for (int j = 0; j < WPW; ++j) {
    const int w = w_first + wave * WPW + j;
    const uint64_t m = __ballot(fb[j] != 0);
    if (lane == 0) {
      cnts[wave * WPW + j] = __popcll(m);
      if (w < nw) words[(size_t)u * nw + w] = m;
    }
  }
  __syncthreads();
  int32_t *bo = blk_off + (size_t)u * (nw + 1);
  int32_t unit_total = 0;
  if (tid == 0) {
    int32_t run = 0;
    for (int i = 0; i < kScanThreads / 64; ++i) run += part[i];
    for (int j = 0; j < kSegWords; ++j) {
      if (w_first + j < nw) bo[w_first + j] = run;
      run += cnts[j];
    }
    if (last_seg) bo[nw] = run;
    unit_total = run;
  }

  plan_tail(plan, num_units, L, u, last_seg, unit_total, arrivals);
}

// The flag scan and the compaction in one launch.  LPR = lanes that share one row (16 bytes each); rows wider than
// 1 KiB loop over segments.  grid = (ceil(nw / 4), units), 4 waves, wave w of workgroup x owns mask word 4 x + w.  A workgroup counts the kept
// tokens before its 256 tokens itself (4 flags per load, at most L bytes, from the caches), so no workgroup waits
// for another and the copy starts one round of loads after the launch instead of after a separate scan kernel.
// It leaves words / blk_off / the prefill plan exactly as ag_flag_scan_kernel does; then a lane's rank inside the
// word plus the word's prefix is the destination row, so the surviving rows are written back-to-back (fully
// coalesced 16-byte stores) and evicted rows are never read.
template <int LPR>
__global__ __launch_bounds__(256) void ag_scan_compact_kernel(const uint8_t *__restrict__ flags, int L, int nw,
                                                              uint64_t *__restrict__ words, int32_t *__restrict__ blk_off,
                                                              ag_pf_plan plan, int num_units, int32_t *__restrict__ arrivals,
                                                              const uint4 *__restrict__ k, const uint4 *__restrict__ v,
                                                              int row_vec, int pos0, uint4 *__restrict__ kc,
                                                              uint4 *__restrict__ vc, int32_t *__restrict__ idx,
                                                              const int64_t *__restrict__ row_off,
                                                              int32_t *__restrict__ len, int32_t *__restrict__ d_err) {
  __shared__ uint8_t sel[4][64];
  __shared__ int32_t cnts[4], part[4];
  const int u = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int w = blockIdx.x * 4 + wave;
  const bool last_seg = blockIdx.x == gridDim.x - 1;
  const uint8_t *f = flags + (size_t)u * L;
  // this wave's flags first (the load is independent of the count below)
  const int t_own = w * 64 + lane;
  const uint8_t f_own = (w < nw && t_own < L) ? f[t_own] : (uint8_t)0;
  // kept tokens before the workgroup's first token
  const int t_end = blockIdx.x * 256;  // <= L
  int before = 0;
  if ((reinterpret_cast<uintptr_t>(f) & 3) == 0) {
    const uint32_t *f4 = reinterpret_cast<const uint32_t *>(f);
    for (int i = tid; i < t_end / 4; i += 256) {
      const uint32_t x = f4[i];
      before += __popc((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u);  // non-zero bytes of x
    }
  } else {
    for (int i = tid; i < t_end; i += 256) before += f[i] != 0;
  }
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o, 64);
  const uint64_t word = __ballot(f_own != 0);
  const int n = __popcll(word);
  if (lane == 0) { part[wave] = before; cnts[wave] = n; }
  __syncthreads();
  int base = part[0] + part[1] + part[2] + part[3];
  for (int i = 0; i < wave; ++i) base += cnts[i];
  int32_t *bo = blk_off + (size_t)u * (nw + 1);
  const int64_t r0 = row_off[u];
  const int64_t cap = row_off[u + 1] - r0;
  int32_t unit_total = 0;
  if (lane == 0 && w < nw) {
    words[(size_t)u * nw + w] = word;
    bo[w] = base;
    if (w == nw - 1) {
      const int total = base + n;
      bo[nw] = total;
      len[u] = (int32_t)(total < cap ? total : cap);
      if (total > cap) atomicOr(d_err, 1);
    }
  }
  if (tid == 0) unit_total = part[0] + part[1] + part[2] + part[3] + cnts[0] + cnts[1] + cnts[2] + cnts[3];
  plan_tail(plan, num_units, L, u, last_seg, unit_total, arrivals);

  // ---- the copy (no workgroup-wide barrier below) ----
  if (w >= nw || n == 0) return;
  const bool keep = (word >> lane) & 1ull;
  const int rank = __popcll(word & ((1ull << lane) - 1ull));
  if (keep) {
    sel[wave][rank] = (uint8_t)lane;
    if (base + rank < cap) idx[r0 + base + rank] = pos0 + w * 64 + lane;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  constexpr int RPI = 64 / LPR;  // rows per wave iteration
  constexpr int UN = 8;          // independent rows in flight per lane group (8: most words need one round of loads)
  const int sub = lane / LPR, seg0 = lane % LPR;
  const size_t src_unit = (size_t)u * L * row_vec;
  // Loads are unconditional (a row index past the word's last kept row re-reads that last row) so that all UN row
  // pairs stay in registers and in flight together; only the stores are predicated.
  for (int c0 = 0; c0 < n; c0 += RPI * UN) {
    size_t src[UN];
#pragma unroll
    for (int j = 0; j < UN; ++j) {
      const int c = c0 + j * RPI + sub;
      src[j] = src_unit + (size_t)(w * 64 + sel[wave][c < n ? c : n - 1]) * row_vec;
    }
    for (int seg = seg0; seg < row_vec; seg += LPR) {
      uint4 kk[UN], vv[UN];
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        kk[j] = k[src[j] + seg];
        vv[j] = v[src[j] + seg];
      }
      // Keeps the compiler from sinking each load into its predicated store, which would serialise the rows.
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        asm volatile("" : "+v"(kk[j].x), "+v"(kk[j].y), "+v"(kk[j].z), "+v"(kk[j].w));
        asm volatile("" : "+v"(vv[j].x), "+v"(vv[j].y), "+v"(vv[j].z), "+v"(vv[j].w));
      }
#pragma unroll
      for (int j = 0; j < UN; ++j) {
        const int c = c0 + j * RPI + sub;
        if (c < n && (int64_t)base + c < cap) {
          const size_t dst = (size_t)(r0 + base + c) * row_vec + seg;
          kc[dst] = kk[j];
          vc[dst] = vv[j];
        }
      }
    }
  }
}

__global__ void ag_slab_offsets_kernel(int64_t *row_off, int units, int L) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u <= units) row_off[u] = (int64_t)u * L;
}

// Packed layout, step 1: kept flags per unit.  grid = units.
__global__ __launch_bounds__(256) void ag_count_kept_kernel(const uint8_t *__restrict__ flags, int L,
                                                            int32_t *__restrict__ kept) {
  __shared__ int32_t part[4];
  const uint8_t *f = flags + (size_t)blockIdx.x * L;
  const int tid = threadIdx.x;
  int n = 0;
  if ((reinterpret_cast<uintptr_t>(f) & 3) == 0) {
    const uint32_t *f4 = reinterpret_cast<const uint32_t *>(f);
    for (int i = tid; i < L / 4; i += 256) {
      const uint32_t x = f4[i];
      n += __popc((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u);  // non-zero bytes of x
    }
    for (int i = (L & ~3) + tid; i < L; i += 256) n += f[i] != 0;
  } else {
    for (int i = tid; i < L; i += 256) n += f[i] != 0;
  }
  for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
  if ((tid & 63) == 0) part[tid >> 6] = n;
  __syncthreads();
  if (tid == 0) kept[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// Packed layout, step 2 (one workgroup): row_off[u + 1] = min(sum_{u' <= u} (kept[u'] + room), total_rows).
__global__ __launch_bounds__(256) void ag_pack_offsets_kernel(const int32_t *__restrict__ kept, int units, int room,
                                                              int64_t total_rows, int64_t *__restrict__ row_off,
                                                              int64_t *__restrict__ rows_needed) {
  __shared__ int64_t wave_sum[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (units + 255) / 256;
  const int u0 = min(units, tid * per), u1 = min(units, u0 + per);
  int64_t sum = 0;
  for (int u = u0; u < u1; ++u) sum += (int64_t)kept[u] + room;
  int64_t incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int64_t up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_sum[wave] = incl;
  __syncthreads();
  int64_t run = incl - sum;
  for (int w = 0; w < wave; ++w) run += wave_sum[w];
  if (tid == 0) row_off[0] = 0;
  for (int u = u0; u < u1; ++u) {
    run += (int64_t)kept[u] + room;
    row_off[u + 1] = run < total_rows ? run : total_rows;
  }
  if (tid == 255 && rows_needed) *rows_needed = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
}

}  // namespace

hipError_t ag_launch_pack_row_off(hipStream_t s, const uint8_t *flags, int units, int L, int room, int64_t total_rows,
                                  int32_t *kept, int64_t *row_off, int64_t *rows_needed) {
  hipLaunchKernelGGL(ag_count_kept_kernel, dim3(units), dim3(256), 0, s, flags, L, kept);
  hipLaunchKernelGGL(ag_pack_offsets_kernel, dim3(1), dim3(256), 0, s, kept, units, room, total_rows, row_off,
                     rows_needed);
  return hipGetLastError();
}

hipError_t ag_launch_slab_offsets(hipStream_t s, int64_t *row_off, int units, int L) {
  hipLaunchKernelGGL(ag_slab_offsets_kernel, dim3((units + 256) / 256), dim3(256), 0, s, row_off, units, L);
  return hipGetLastError();
}

size_t ag_ws_scan_bytes(int units, int L) {
  const size_t nw = ag_nwords(L);
  return ag_align256((size_t)units * nw * sizeof(uint64_t)) + ag_align256((size_t)units * (nw + 1) * sizeof(int32_t));
}

hipError_t ag_launch_flag_scan(ag_ctx *ctx, hipStream_t s, const uint8_t *flags, int units, int L, uint64_t *words,
                               int32_t *blk_off, const ag_pf_plan *plan) {
  const int nw = ag_nwords(L);
  ag_pf_plan none;
  memset(&none, 0, sizeof(none));
  int32_t *arrivals = ctx->d_err + 16;  // zeroed at creation; the kernel leaves it at zero
  AG_LAUNCH(ag_time_kernel(ctx, AG_K_FLAG_SCAN), ag_flag_scan_kernel, dim3((nw + kSegWords - 1) / kSegWords, units),
            dim3(kScanThreads), 0, s, flags, L, nw, words, blk_off, plan ? *plan : none, units, arrivals);
  return hipGetLastError();
}

hipError_t ag_launch_scan_compact(ag_ctx *ctx, hipStream_t s, const uint8_t *flags, int units, int L, uint64_t *words,
                                  int32_t *blk_off, const ag_pf_plan *plan, const void *k, const void *v, int row_bytes,
                                  int pos0, void *kc, void *vc, int32_t *idx, const int64_t *row_off, int32_t *len) {
  const int nw = ag_nwords(L);
  const int row_vec = row_bytes / 16;
  ag_pf_plan none;
  memset(&none, 0, sizeof(none));
  int32_t *arrivals = ctx->d_err + 16;  // zeroed at creation; the kernel leaves it at zero
  const dim3 grid((nw + 3) / 4, units), block(256);
#define AG_SC(LPR)                                                                                                  \
  AG_LAUNCH(ev, ag_scan_compact_kernel<LPR>, grid, block, 0, s, flags, L, nw, words, blk_off, plan ? *plan : none, \
                     units, arrivals, (const uint4 *)k, (const uint4 *)v, row_vec, pos0, (uint4 *)kc, (uint4 *)vc, idx, \
                     row_off, len, ctx->d_err)
  const ag_evpair ev = ag_time_kernel(ctx, AG_K_COMPACT);
  if (row_vec <= 8) AG_SC(8);
  else if (row_vec <= 16) AG_SC(16);
  else if (row_vec <= 32) AG_SC(32);
  else AG_SC(64);
#undef AG_SC
  return hipGetLastError();
}
