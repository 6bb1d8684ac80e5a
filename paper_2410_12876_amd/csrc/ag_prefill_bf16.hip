// Flag-masked causal prefill attention (Eq. 2 under the mask of Eq. 5), bf16, head dimension 128 -- the
// tuned CDNA4 kernel.  Same formulation as ag_prefill.hip (attention over the compacted rows with a per-query
// boundary: cnt[j] + 1 rows for a kept token, whose own row is cache row cnt[j]; cnt[j] rows plus its own
// key/value from the uncompacted tensors, which initialise the online softmax, for an evicted one), built for gfx950:
//
//   * K and V tiles (64 cache rows x 256 B) go from global memory straight into LDS (buffer_load ... lds,
//     no register staging), double-buffered, one workgroup barrier per step.
//   * Both tiles stay row-major in LDS.  The 16-byte chunk index of a row is XOR-swizzled with a bit-swapped
//     row nibble, applied on the global-address side of the load, so that the 128-bit reads of K fragments
//     (32 consecutive rows, same column) and the transposing reads of V fragments (4 consecutive rows,
//     64 contiguous bytes each) are both free of bank conflicts (SQ_LDS_BANK_CONFLICT reads 0).
//   * V is never transposed in memory: ds_read_b64_tr_b16 delivers, per lane, four consecutive keys of one
//     head-dim column, which is the A-operand layout of O^T += V^T . P^T.
//   * A lane owns one query: S^T = K . Q^T and O^T = V^T . P^T on v_mfma_f32_32x32x16_bf16, P packed with
//     v_cvt_pk_bf16_f32 straight from the S^T accumulators, row max / sum / rescale as per-lane scalars.
//   * The reference maximum is only raised (and O rescaled) when a row's new maximum exceeds it by more than
//     2^8; otherwise the stale maximum is kept, which is exact after the final division by the row sum.
//   * Software pipeline: S^T of the next tile is issued while the softmax of the current tile runs.
//   * Small launches (one 4096-token layer is ~1000 workgroups of very different length) are bounded by
//     their longest workgroup, the last query tile of the head that keeps most.  There the key range of a
//     (head, query tile) item is cut into chunks of at most `chunk_tiles` tiles, one workgroup per chunk;
//     chunk_tiles is a little above the average number of tiles per workgroup slot, measured on the device from
//     the flags, so only an item that alone exceeds it is cut.  Items that fit one chunk write their output
//     directly; the few long ones store unnormalised fp32 partial states in the workspace, and the chunk that
//     arrives last (a per-item counter) combines them, in an order that does not depend on who is last, and writes
//     the rows.
//   * Query rows come in and output rows go out as whole 256-byte rows (4 rows per instruction), turned into and
//     out of the per-lane fragment layout through LDS; the scattered 16- and 8-byte pieces of the fragment layout
//     would cost the texture path several times the address cycles.
//   * Workgroups go to the 8 XCDs, and inside an XCD to its 4 shader engines, round-robin by their index
//     (measured: workgroup i runs on XCD i % 8, engine (i / 8) % 4), so the index -> (head, query tile) map
//     decides both L2 locality and balance.  All tiles of one head are given to one XCD (its K/V stay in that
//     XCD's L2), longest first; the flag scan's last workgroup first deals the heads to the XCDs in
//     snake order of their kept-row counts, and the heads of an XCD rotate over its engines from one query tile
//     to the next, so every engine gets about the same number of key tiles although heads keep 20 % to 90 %.
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "ag_prefill_bf16_common.h"


namespace {

// GB = query heads of one KV group per workgroup (one per wave).  n_split = chunks per item in the grid,
// chunk_tiles_dev = key tiles per chunk (device value, NULL without a split); part = partial states
// [item][chunk][4 waves][66][64] fp32 and tickets = per-item arrival counters (n_split > 1).
// BAND = the recent-token variant (Table 6 of the appendix): the evicted tokens among the n_recent - 1 tokens just before a query
// stay visible to it.  They are read from the uncompacted K/V as up to three extra 64-key "band" tiles that run
// through the same pipeline ahead of the compacted tiles of chunk 0, with their own mask.
// NW = waves per workgroup: 4 (two workgroups per CU).  (8, one workgroup per CU with twice the queries sharing
// every K/V tile, also works without the band variant but is slower: the whole CU then moves in step.)
template <int D, int GB, bool BAND, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void ag_prefill_bf16_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint64_t *__restrict__ words, const int32_t *__restrict__ blk_off, const uint16_t *__restrict__ kc,
    const uint16_t *__restrict__ vc, const int64_t *__restrict__ row_off, int L, int Hq, int Hkv, int nw, int n_hy,
    int n_split, int n_sp, const int32_t *__restrict__ chunk_tiles_dev, float qscale, int n_recent,
    const int32_t *__restrict__ order, int head_major, uint16_t *__restrict__ out, int out_token_major,
    float *__restrict__ part, int32_t *__restrict__ tickets) {
  typedef pf_geom<D> geo;
  constexpr int kRowB = geo::kRowB, kTileB = geo::kTileB, kGroupB = geo::kGroupB;
  constexpr int CPR = geo::CPR;  // 16-byte chunks per row: 16 (D = 128) or 8 (D = 64)
  constexpr int RPI = geo::RPI;  // rows per load or store instruction: 4 or 8
  auto swz = [](int r) { return geo::swz(r); };
  constexpr int QW = NW / GB;  // query sub-tiles per workgroup
  constexpr int RPW = kBN / NW;  // tile rows each wave loads
  constexpr int LI = RPW / RPI;  // load instructions per wave and tile (RPI rows each)
  constexpr int BM = 32 * QW;  // queries per workgroup
  constexpr int KS = D / 16;   // k-steps of S^T
  constexpr int DT = D / 32;   // 32-row tiles of O^T
  __shared__ __attribute__((aligned(1024))) uint8_t smem[kGroupB];  // [K0][K1][V0][V1], each [row][256 B]
  // BAND: per band tile, the rows whose value row held a NaN or an infinity (see scrub_band_v below)
  __shared__ uint32_t nf_rows[BAND ? 3 : 1][2];

  const int G = Hq / Hkv;
  const int HB = G / GB;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar, so that LDS bases stay in SGPRs
  const int w4 = wave;
  const int col = lane & 31, hb = lane >> 5;
  // workgroup id -> (query tile, chunk, unit/head block): heads vary fastest so that a head keeps its XCD
  const int n_qt = (L + BM - 1) / BM;
  // The first n_sp rows of query tiles (the longest) have n_split workgroups per item, one per key chunk; a shorter
  // row cannot hold an item of more than one chunk (a chunk is never shorter than max_tiles / n_split tiles) and has
  // one workgroup per item.
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
    // Many heads: the resident workgroups should cover few of them, or a head's K/V rows leave the L2 between
    // two of its query tiles and every tile comes from HBM again.  XCD x (workgroups x, x + 8, ...) walks heads
    // x, x + 8, ... one after the other, each head's query tiles together, longest first.
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
    rem = (j / n_qt) * 8 + x;
    qt_idx = j % n_qt;
    if (rem >= n_hy) return;  // the grid is rounded up to whole groups of 8 heads
  }
  const int qtile = n_qt - 1 - qt_idx;  // longest rows first
  // Position pos of a row goes to XCD pos % 8 and, inside it, to shader engine (pos / 8) % 4: both fixed for all
  // rows.  order[] gives each XCD its heads; rotating them over the XCD's positions from row to row lets every
  // shader engine see all of them, instead of one engine being stuck with the head that keeps most.
  const int pos = rem % n_hy;
  int hy = pos;
  if (order && !head_major) {
    const int n_slot = n_hy >> 3;
    hy = order[(((pos >> 3) + qt_idx) % n_slot) * 8 + (pos & 7)];
  }
  const int u = hy / HB;
  const int hblk = hy - u * HB;
  const int b = u / Hkv, g = u - b * Hkv;
  const int head = g * G + hblk * GB + (w4 % GB);
  const int j0 = qtile * BM + (w4 / GB) * 32;
  const int jq = min(j0 + col, L - 1);

  // All scalar inputs of the workgroup in one round of loads.  The 32 queries of a wave lie in one 64-token
  // mask word (j0 is a multiple of 32), so one (word, prefix) pair gives every per-query boundary of the wave.
  const uint64_t *wu = words + (size_t)u * nw;
  const int32_t *bo = blk_off + (size_t)u * (nw + 1);
  const int jw = min(j0, L - 1) >> 6;                         // mask word of this wave's queries
  const int jb = min(qtile * BM + BM - 1, L - 1);             // last query of the workgroup
  const uint64_t word_w = wu[jw], word_b = wu[jb >> 6];
  const int pre_w = bo[jw], pre_b = bo[jb >> 6], kept_u = bo[nw];
  const int chunk_tiles = chunk_tiles_dev ? *chunk_tiles_dev : 0x7fffffff / kBN;
  const int64_t ro0 = row_off[u], ro1 = row_off[u + 1];
  auto cnt_in = [](uint64_t w, int pre, int j) { return pre + __popcll(w & ((1ull << (j & 63)) - 1ull)); };
  const int len_u = (int)min((int64_t)kept_u, ro1 - ro0);
  // A kept token's own key and value are row cnt(j) of the compacted rows, so its visible set is simply the first
  // cnt(j) + 1 of them; only an evicted token (or one whose row did not fit the cache) takes its own k, v from the
  // uncompacted tensors.  bnd = number of compacted rows query j sees.
  auto in_cache = [&](uint64_t w, int pre, int j) { return ((w >> (j & 63)) & 1ull) != 0 && cnt_in(w, pre, j) < len_u; };
  auto bnd_in = [&](uint64_t w, int pre, int j) { return cnt_in(w, pre, j) + (in_cache(w, pre, j) ? 1 : 0); };
  // (all boundaries are clamped to the rows the cache holds: after a capacity overflow the rows that did not fit
  // are simply not there -- their tokens count as evicted -- and nothing past len_u is attended)
  const int cnt_q = min(bnd_in(word_w, pre_w, jq), len_u);
  const bool own_kv = chunk == 0 && !in_cache(word_w, pre_w, jq);  // this query's diagonal term comes from k, v
  const int cnt_wave_lo = min(bnd_in(word_w, pre_w, min(j0, L - 1)), len_u);
  const int cnt_wave_hi = j0 < L ? min(bnd_in(word_w, pre_w, min(j0 + 31, L - 1)), len_u) : 0;
  const int cnt_blk = min(bnd_in(word_b, pre_b, jb), len_u);
  const int n_tiles = (cnt_blk + kBN - 1) / kBN;       // key tiles of the item
  const int tile0 = chunk > 0 ? chunk * chunk_tiles : 0;  // this workgroup's chunk: tiles [tile0, tile0 + n_steps)
  if (chunk > 0 && tile0 >= n_tiles) return;           // empty chunk (the whole workgroup leaves)
  const int n_chunks = max(1, (n_tiles + chunk_tiles - 1) / chunk_tiles);
  // band tiles (chunk 0 only): 64-aligned tiles of original token positions that can hold a key of this
  // workgroup's queries, i.e. positions [first query - (n_recent - 1), last query - 1]
  int n_band = 0, band_t0 = 0;
  uint64_t bw0 = 0, bw1 = 0, bw2 = 0;  // keep masks of the band tiles
  if (BAND && chunk == 0) {
    const int klo = max(0, qtile * BM - (n_recent - 1)), khi = jb - 1;
    if (khi >= klo) {
      band_t0 = klo >> 6;
      n_band = (khi >> 6) - band_t0 + 1;  // <= 3 because n_recent <= 64 and BM <= 128
      // keep bits of the tokens that are among the compacted rows: all kept ones, unless the cache overflowed --
      // a kept token that found no room is not there, so the band must show it like an evicted one
      auto in_cache_bits = [&](int t) {
        uint64_t w = wu[t];
        const int room = len_u - bo[t];
        if (room <= 0) return (uint64_t)0;
        while (__popcll(w) > room) w &= ~(1ull << (63 - __clzll(w)));  // (never entered without an overflow)
        return w;
      };
      bw0 = in_cache_bits(band_t0);
      if (n_band > 1) bw1 = in_cache_bits(band_t0 + 1);
      if (n_band > 2) bw2 = in_cache_bits(band_t0 + 2);
    }
  }
  // steps of this workgroup: the band tiles first, then its chunk of compacted tiles
  const int n_steps = n_band + max(0, min(n_tiles - tile0, chunk_tiles));
  if (BAND && tid < 6) nf_rows[tid >> 1][tid & 1] = 0u;  // ordered before its first use by the barrier ahead of step 0

  const uint16_t *Kc = kc + (size_t)ro0 * D;
  const uint16_t *Vc = vc + (size_t)ro0 * D;

  // ---- tile loader: wave w4 of a group fills rows [16 w4, 16 w4 + 16) of the group's K and V tiles, 4 rows
  // (1 KiB) per instruction.  lane -> (row r = 16 w4 + 4 i + lane/16, physical chunk p = lane%16); it fetches
  // logical chunk p ^ swz(r).  Buffer loads with the LDS modifier: the descriptor ends at the unit's last
  // valid row, so rows past the end arrive as zeros (their scores are masked anyway) and nothing outside the
  // unit's slab is ever read.  The loads are issued from inline assembly so that the compiler does not
  // serialise later LDS reads of the *other* buffer behind them; completion is awaited explicitly
  // (s_waitcnt vmcnt(0)) before the barrier that publishes the tile.
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Kc, 0, len_u * kRowB, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Vc, 0, len_u * kRowB, 0x00020000);
  // the unit's uncompacted rows (band tiles); rows past the prompt's end arrive as zeros and are masked
  const __amdgpu_buffer_rsrc_t kb_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)(k + (size_t)u * L * D), 0, BAND ? L * kRowB : 0, 0x00020000);
  const __amdgpu_buffer_rsrc_t vb_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)(v + (size_t)u * L * D), 0, BAND ? L * kRowB : 0, 0x00020000);
  const int ld_r = lane / CPR;
  int ld_off[LI];
#pragma unroll
  for (int i = 0; i < LI; ++i) {
    const int r = RPW * w4 + RPI * i + ld_r;
    ld_off[i] = r * kRowB + (((lane % CPR) ^ swz(r)) << 4);  // chunk (lane % CPR) ^ swz(r)
  }
  const uint32_t ld_base = (uint32_t)(size_t)((AG_LDS uint8_t *)smem) + w4 * RPW * kRowB;
  auto issue_k = [&](int i_step) {  // K of the tile of step i_step -> K buffer i_step & 1
    const bool bnd = BAND && i_step < n_band;
    const int soff = (bnd ? band_t0 + i_step : tile0 + i_step - n_band) * kTileB;
    const __amdgpu_buffer_rsrc_t rsrc = bnd ? kb_rsrc : k_rsrc;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const uint32_t dk = ld_base + (i_step & 1) * kTileB + i * RPI * kRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dk), "v"(ld_off[i]), "s"(rsrc), "s"(soff) : "memory");
    }
  };
  auto issue_v = [&](int i_step) {
    const bool bnd = BAND && i_step < n_band;
    const int soff = (bnd ? band_t0 + i_step : tile0 + i_step - n_band) * kTileB;
    const __amdgpu_buffer_rsrc_t rsrc = bnd ? vb_rsrc : v_rsrc;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const uint32_t dv = ld_base + 2 * kTileB + (i_step & 1) * kTileB + i * RPI * kRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dv), "v"(ld_off[i]), "s"(rsrc), "s"(soff) : "memory");
    }
  };
  if (n_steps > 0) { issue_k(0); issue_v(0); }
  if (n_steps > 1) issue_k(1);

  // ---- Q fragments (B operand of S^T): lane (query col, half hb), k-step ks: Q[j][16 ks + 8 hb .. +8); for chunk 0
  // also the query's own key row (same layout) and value row (lane: d = 32 dt + 8 r4 + 4 hb .. +4) ----
  // A lane needs 16-byte pieces of ITS query's row, so direct loads would touch 64 different cache lines per
  // instruction (measured: 4.5 us of a workgroup's 7 us start-up).  Instead the wave reads its 32 rows with
  // whole-line loads (lane -> row 4 j + lane/16, 16-byte chunk lane%16: 1 KiB contiguous per instruction) and turns
  // them into fragments through a private 4 KiB corner of the V1 tile buffer, 16 rows at a time; V1 is not a
  // load target before the first step.  Chunks are XOR-swizzled with the row so that both sides are conflict-free.
  uint4 qf[KS], kself[KS];
  uint2 vself[DT][4];
  {
    const int srow = lane / CPR, schunk = lane % CPR;
    constexpr int RP = (kTileB / NW) / kRowB;  // rows per pass: the wave's corner of V1 holds RP whole rows
    constexpr int NP = 32 / RP;                // passes
    constexpr int LP = RP / RPI;               // whole-row loads per pass (RPI rows each)
    u32x4 sq[NP][LP], sk[NP][LP], sv[NP][LP];
#pragma unroll
    for (int h = 0; h < NP; ++h)
#pragma unroll
      for (int j = 0; j < LP; ++j) {
        const int row = min(j0 + RP * h + RPI * j + srow, L - 1);
        // All three loads are unconditional (conditional ones end up in scratch memory).  A row whose k, v are not
        // needed -- a kept token, or any row in a later chunk of a split item -- is pointed at the wave's first row
        // instead, which costs one cache line per wave instead of HBM traffic per row.
        const int kv_row = (chunk == 0 && !in_cache(word_w, pre_w, row)) ? row : min(j0, L - 1);
        sq[h][j] = *reinterpret_cast<const u32x4 *>(q + ((size_t)(b * Hq + head) * L + row) * D + 8 * schunk);
        sk[h][j] = *reinterpret_cast<const u32x4 *>(k + ((size_t)u * L + kv_row) * D + 8 * schunk);
        sv[h][j] = *reinterpret_cast<const u32x4 *>(v + ((size_t)u * L + kv_row) * D + 8 * schunk);
      }
    AG_LDS uint8_t *stage = (AG_LDS uint8_t *)smem + 3 * kTileB + w4 * (kTileB / NW);
    const int rr = col % RP;  // this lane's row inside a pass
    const int rk = geo::key(rr);
    // lanes exchange data through the corner: a wave-level release/acquire pair on each side tells the compiler
    // that one lane's store is another lane's load (the hardware keeps a wave's LDS accesses in order anyway)
    auto wave_sync = [] {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto put = [&](const u32x4 (&x)[LP]) {
      wave_sync();  // the previous contents have been read
#pragma unroll
      for (int j = 0; j < LP; ++j) {
        const int r = RPI * j + srow;
        *reinterpret_cast<AG_LDS u32x4 *>(stage + r * kRowB + ((schunk ^ geo::key(r)) << 4)) = x[j];
      }
      wave_sync();  // the rows are there for every lane
    };
    auto get4 = [&](int off) {
      const u32x4 x = *reinterpret_cast<const AG_LDS u32x4 *>(stage + off);
      return make_uint4(x[0], x[1], x[2], x[3]);
    };
#pragma unroll
    for (int h = 0; h < NP; ++h) {
      const bool mine = (col / RP) == h;
      put(sq[h]);
      if (mine) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          qf[ks] = get4(rr * kRowB + (((2 * ks + hb) ^ rk) << 4));
      }
      if (chunk == 0) {
        put(sk[h]);
        if (mine) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            kself[ks] = get4(rr * kRowB + (((2 * ks + hb) ^ rk) << 4));
        }
        put(sv[h]);
        if (mine) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
            {
              const u32x2 x = *reinterpret_cast<const AG_LDS u32x2 *>(stage + rr * kRowB + (((4 * dt + r4) ^ rk) << 4) + 8 * hb);
              vself[dt][r4] = make_uint2(x[0], x[1]);
            }
        }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the corner is read out before anyone may load V(1) over it
  }
  __builtin_amdgcn_sched_barrier(0);  // keep the loads above ahead of the arithmetic below

  // ---- initial online-softmax state: chunk 0 starts from the query's own token, the others from nothing ----
  float m_run = kEmptyMax;  // reference maximum of the exponentials, log2 units
  float l_run = 0.f;        // each half (hb) of a column holds part of the row sum
  f32x16 acc_o[DT];         // O^T: acc_o[dt][r] = (d = 32 dt + 8 (r/4) + 4 hb + r%4, query col)
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[dt][r] = 0.f;
  if (chunk == 0) {
    float s_self = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint32_t qa[4] = {qf[ks].x, qf[ks].y, qf[ks].z, qf[ks].w};
      const uint32_t ka[4] = {kself[ks].x, kself[ks].y, kself[ks].z, kself[ks].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s_self = fmaf(__uint_as_float(qa[e] << 16), __uint_as_float(ka[e] << 16), s_self);
        s_self = fmaf(__uint_as_float(qa[e] & 0xffff0000u), __uint_as_float(ka[e] & 0xffff0000u), s_self);
      }
    }
    s_self += __shfl_xor(s_self, 32, 64);
    // (selects, not arithmetic: what was loaded for a query that does not use it may be anything)
    m_run = own_kv ? s_self * qscale : kEmptyMax;
    l_run = own_kv && hb == 0 ? 1.f : 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        acc_o[dt][4 * r4 + 0] = own_kv ? __uint_as_float(vself[dt][r4].x << 16) : 0.f;
        acc_o[dt][4 * r4 + 1] = own_kv ? __uint_as_float(vself[dt][r4].x & 0xffff0000u) : 0.f;
        acc_o[dt][4 * r4 + 2] = own_kv ? __uint_as_float(vself[dt][r4].y << 16) : 0.f;
        acc_o[dt][4 * r4 + 3] = own_kv ? __uint_as_float(vself[dt][r4].y & 0xffff0000u) : 0.f;
      }
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

  const AG_LDS uint8_t *lds_grp = (const AG_LDS uint8_t *)smem;
  auto s_tile = [&](int i_step, f32x16 (&acc)[2]) {  // acc = K(tile of step i_step) . Q^T
    const AG_LDS uint8_t *Kt = lds_grp + (i_step & 1) * kTileB;
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
  // Softmax of one tile held in acc (key = c0 + 32 sub + 8 (r/4) + 4 hb + r%4, query = col) -> pf, l_run, m_run.
  // The matrix pipe and the vector ALU share the wave's issue slots, so every vector instruction per element counts;
  // the common case is therefore three per element and a half: one fused multiply-add (scale, minus the reference
  // maximum), one exponential, half a pack, half a dot2 that sums the PACKED pair -- the row sum is then the sum of
  // exactly the bf16 weights the second MFMA multiplies with.  No maximum is taken there: the exponentials are formed
  // against the reference maximum as it stands, and only if a lane's sum of weights then exceeds 2^kLazyLog2 (or is
  // not a number: the first tile, whose reference is still "nothing seen") does the wave take the slow branch, which
  // finds the row maxima, raises the references that need it and forms the weights again.  A stale reference is
  // exact after the final division by the row sum -- floating point is indifferent to the common factor -- and
  // 2^kLazyLog2 times the 64 keys of a tile times the tiles of the longest prompt stays far inside fp32's range.
  // A lane raises its own reference only (its pair lane^32 decides with it), so a query never depends on the
  // queries that share its wave.
  float psum;
  auto weights = [&](f32x16 (&acc)[2]) {
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    psum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(fmaf(acc[sub][r], qscale, -m_run));
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        pf[sub][sl] = make_uint4(pack2(p[8 * sl + 0], p[8 * sl + 1]), pack2(p[8 * sl + 2], p[8 * sl + 3]),
                                 pack2(p[8 * sl + 4], p[8 * sl + 5]), pack2(p[8 * sl + 6], p[8 * sl + 7]));
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[sub][sl].x), ones, psum, false);
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[sub][sl].y), ones, psum, false);
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[sub][sl].z), ones, psum, false);
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf[sub][sl].w), ones, psum, false);
      }
    }
  };
  auto softmax_tile = [&](f32x16 (&acc)[2]) {  // the common case; sets any_raise when softmax_raise must follow
    weights(acc);
    alpha_pending = 1.f;
    any_raise = __any(!(psum <= kLazyLimit));
  };
  auto softmax_raise = [&](f32x16 (&acc)[2]) {  // rare: some row of the wave outgrew its reference maximum
    const uint64_t big = __ballot(!(psum <= kLazyLimit));
    const bool mine = (((big | (big >> 32) | (big << 32)) >> lane) & 1ull) != 0;  // this lane's query, either half
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[sub][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * qscale;
    const float m_new = mine && mx > m_run ? mx : m_run;   // (selects: the others keep their reference and factor 1)
    alpha_pending = mine && mx > m_run ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
    m_run = m_new;
    weights(acc);
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
  // band tile of step i: key position t = 64 (band_t0 + i) + kk is visible to query jq iff it lies among the
  // n_recent - 1 positions before jq and its keep bit is clear (kept tokens are among the compacted rows)
  auto band_mask = [&](int i, f32x16 (&acc)[2]) {
    const int r0 = (band_t0 + i) * kBN;
    const uint64_t bword = i == 0 ? bw0 : (i == 1 ? bw1 : bw2);
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      // this lane's keys of the sub-tile are 32 sub + 4 hb + c with c = 8 (r/4) + r%4: one 32-bit slice of the keep
      // mask and one distance, then compile-time shifts per element
      const uint32_t wsub = (uint32_t)(bword >> (32 * sub + 4 * hb));
      const int dl = jq - 1 - r0 - 32 * sub - 4 * hb;  // (query - 1) - key for c = 0
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int c = 8 * (r >> 2) + (r & 3);
        const bool in_window = (unsigned)(dl - c) < (unsigned)(n_recent - 1);  // query - n_recent < key < query
        if (!in_window || ((wsub >> c) & 1u)) acc[sub][r] = -INFINITY;
      }
    }
  };
  // does step i hold a key that some query of this wave may see?  (wave-uniform)
  auto vis = [&](int i) -> bool {
    if (BAND && i < n_band) {
      const int r0 = (band_t0 + i) * kBN;
      return j0 < L && r0 <= j0 + 30 && r0 + kBN - 1 >= j0 - (n_recent - 1);
    }
    return (tile0 + i - n_band) * kBN < cnt_wave_hi;
  };
  auto pv_tile = [&](int i_step) {  // O^T += V(tile)^T . P^T, after the pending rescale
    if (any_raise) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha_pending;
    }
    const AG_LDS uint8_t *Vt = lds_grp + 2 * kTileB + (i_step & 1) * kTileB;
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
    for (int i = 0; i < 4 * DT; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
      if (i < 4 * DT - 4) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
  };
  // Band tiles hold rows this workgroup's queries must not see (kept tokens, tokens outside a query's window) next
  // to rows they do see.  Their scores are replaced by -inf by a select, so K may hold anything there; but in
  // O^T += V^T . P^T a weight of exactly 0 still meets the masked row's values, and 0 x NaN is NaN.  So every wave
  // scrubs the value rows it loaded itself before the tile is published: a row with a NaN or an infinity in it is
  // zeroed in LDS and noted in nf_rows; a query that does see such a row (its window mask meets nf_rows) gets NaN
  // as its whole output row -- what the planted value would have given it -- and nobody else is touched.
  bool poisoned = false;
  auto scrub_band_v = [&](int i) {
    AG_LDS uint8_t *vt = (AG_LDS uint8_t *)smem + 2 * kTileB + (i & 1) * kTileB + w4 * RPW * kRowB + lane * 16;
#pragma unroll
    for (int ii = 0; ii < LI; ++ii) {
      const u32x4 x = *reinterpret_cast<const AG_LDS u32x4 *>(vt + ii * RPI * kRowB);
      bool bad = false;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        bad |= (x[e] & 0x7f80u) == 0x7f80u || (x[e] & 0x7f800000u) == 0x7f800000u;
      const uint32_t row_bad = (uint32_t)(__ballot(bad) >> (CPR * ld_r)) & ((1u << CPR) - 1u);  // the CPR lanes of my row
      if (row_bad) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<AG_LDS u32x4 *>(vt + ii * RPI * kRowB) = z;
        const int r = RPW * w4 + RPI * ii + ld_r;
        if ((lane % CPR) == 0) atomicOr(&nf_rows[i][r >> 5], 1u << (r & 31));
      }
    }
  };
  // keys of band tile i (bit kk = position 64 (band_t0 + i) + kk) that query jq sees through its window
  auto band_visible = [&](int i) -> uint64_t {
    const int r0 = (band_t0 + i) * kBN;
    const uint64_t bword = i == 0 ? bw0 : (i == 1 ? bw1 : bw2);
    const int lo = max(0, jq - (n_recent - 1) - r0), hi = min(kBN - 1, jq - 1 - r0);
    if (hi < lo) return 0ull;
    const uint64_t win = (hi - lo == 63 ? ~0ull : ((1ull << (hi - lo + 1)) - 1ull)) << lo;
    return win & ~bword;
  };
  // One pipeline step.  cur holds S^T of this group's tile of step i; nxt receives that of step i + 1.
  // At the top (after the barrier) K(i+1) and V(i) are resident; the step then requests K(i+2) into the K
  // buffer that step i used and V(i+1) into the V buffer of step i-1.
  auto step = [&](int i, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of K(i+1), V(i) has landed
    if (BAND && i < n_band) scrub_band_v(i);
    __syncthreads();                                  // ... and everyone's; step i-1 is fully consumed
    if (i + 2 < n_steps) issue_k(i + 2);
    if (i + 1 < n_steps) issue_v(i + 1);
    const int c0 = (tile0 + i - n_band) * kBN;
    const bool vis_cur = vis(i);                                                 // wave-uniform
    const bool vis_nxt = i + 1 < n_steps && vis(i + 1);                          // wave-uniform
    if (vis_cur) {
      if (BAND && i < n_band) {
        band_mask(i, cur);
        const uint64_t nf = ((uint64_t)nf_rows[i][1] << 32) | nf_rows[i][0];
        poisoned |= (band_visible(i) & nf) != 0ull;
      } else {
        mask_tile(c0, cur);
      }
    }
    if (BAND && vis_nxt && !vis_cur) {
      s_tile(i + 1, nxt);   // band tiles are not all visible to a wave: the next tile may be the first it sees
    } else if (vis_nxt) {
      s_tile(i + 1, nxt);   // MFMA stream ...
      softmax_tile(cur);    // ... and an independent VALU stream; the groups below interleave them:
      // 4 K-fragment reads ahead, then per MFMA one more read and a slice of the softmax arithmetic
      constexpr int NM = 2 * KS, AHEAD = NM / 4;  // MFMAs of S^T; fragment reads issued ahead of them
      __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
      for (int n = 0; n < NM; ++n) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (n < NM - AHEAD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 96 / NM, 0);
      }
      if (any_raise) softmax_raise(cur);
    } else if (vis_cur) {
      softmax_tile(cur);
      if (any_raise) softmax_raise(cur);
    }
    if (vis_cur) {
      l_run = l_run * alpha_pending + psum;
      pv_tile(i);
    }
  };
  f32x16 acc_a[2], acc_b[2];
  if (n_steps > 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (vis(0)) s_tile(0, acc_a);
  }
  for (int i = 0; i < n_steps; i += 2) {
    step(i, acc_a, acc_b);
    if (i + 1 < n_steps) step(i + 1, acc_b, acc_a);
  }

  if (BAND && poisoned) l_run = __builtin_nanf("");  // survives the merge of chunk states and the final division
  // ---- an item cut into chunks: store this chunk's state; the chunk that arrives last merges and writes ----
  if (n_chunks > 1) {
    const size_t item = (size_t)qtile * n_hy + hy;
    float *st = part + (item * n_split * NW + w4) * geo::kState + lane;  // state of chunk c at st + c * cstride
    const size_t cstride = (size_t)NW * geo::kState;
    // The states travel through memory between workgroups of one launch.  They are written through and read
    // past the caches (system-scope relaxed accesses), so no cache-wide write-back or invalidate is needed: the
    // stores are complete (vmcnt 0) before the workgroup's arrival is counted, and the last arrival reads after it.
    float *mine = st + chunk * cstride;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        __hip_atomic_store(&mine[(16 * dt + r) * 64], acc_o[dt][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&mine[16 * DT * 64], m_run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&mine[(16 * DT + 1) * 64], l_run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // every wave's state is out, and nobody reads the tile buffers any more
    int *last = reinterpret_cast<int *>(smem);
    if (tid == 0)
      *last = __hip_atomic_fetch_add(&tickets[item], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_chunks - 1;
    __syncthreads();
    if (!*last) return;
    auto peek = [](const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); };
    float m = m_run;
    for (int c = 0; c < n_chunks; ++c)
      if (c != chunk) m = fmaxf(m, peek(&st[c * cstride + 16 * DT * 64]));
    // Rounded product + rounded product (never a fused multiply-add), so that the result does not depend on which chunk
    // arrives last: two chunks are one commutative addition of this chunk's registers and the other's state; more
    // are added in chunk order starting from zero, this chunk's own state read back like the others'.
    if (n_chunks == 2) {
      const float f_own = __builtin_amdgcn_exp2f(m_run - m);
      l_run = mul_round(l_run, f_own);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] = mul_round(acc_o[dt][r], f_own);
    } else {
      l_run = 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] = 0.f;
    }
    for (int c = 0; c < n_chunks; ++c) {
      if (n_chunks == 2 && c == chunk) continue;
      const float *sc = st + c * cstride;
      const float f = __builtin_amdgcn_exp2f(peek(&sc[16 * DT * 64]) - m);
      l_run = mul_round_add(peek(&sc[(16 * DT + 1) * 64]), f, l_run);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] = mul_round_add(peek(&sc[(16 * dt + r) * 64]), f, acc_o[dt][r]);
    }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  // Output rows leave as whole 256-byte rows.  A lane owns one query and 4-element pieces of its row, so direct
  // stores would be 16 instructions of 64 scattered 8-byte pieces each; instead the wave lays its 32 rows out in
  // 8 KiB of the (now unused) tile buffers, 16-byte chunks XOR-swizzled with the row, and stores them with 8
  // instructions of 4 whole rows each (lane -> row 4 i + lane / 16, chunk lane % 16).
  __syncthreads();  // every wave is done with the K/V tiles
  {
    AG_LDS uint8_t *ost = (AG_LDS uint8_t *)smem + w4 * (32 * kRowB);
    // (the lane number is laundered through an empty asm so that the addresses below are computed here, from one
    // register, instead of being shared with the look-alike ones of the query staging and kept alive -- in spill
    // slots, for the recent-token variant -- across the whole tile loop)
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int col_e = lane_e & 31, hb_e = lane_e >> 5;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const u32x2 o = {pack2(acc_o[dt][4 * r4 + 0] * inv, acc_o[dt][4 * r4 + 1] * inv),
                         pack2(acc_o[dt][4 * r4 + 2] * inv, acc_o[dt][4 * r4 + 3] * inv)};
        *reinterpret_cast<AG_LDS u32x2 *>(ost + col_e * kRowB + (((4 * dt + r4) ^ geo::key(col_e)) << 4) + 8 * hb_e) = o;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // one lane's store is another lane's load
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // head-major [B, Hq, L, D] like q, or token-major [B, L, Hq, D] (heads of a token side by side): the wave's rows
    // start at a wave-uniform address and lie row_stride apart
    const int row_stride = (out_token_major ? Hq : 1) * kRowB;
    uint16_t *obase = out + (out_token_major ? (((size_t)b * L + j0) * Hq + head) * D : ((size_t)(b * Hq + head) * L + j0) * D);
    const int n_rows = min(32, L - j0);  // <= 0 for a wave past the end of the prompt: nothing is stored
    const __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)obase, 0, n_rows > 0 ? (uint32_t)((n_rows - 1) * row_stride + kRowB) : 0u, 0x00020000);
    const int orow_l = lane_e / CPR, ochunk = lane_e % CPR;
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
      const int row = RPI * i + orow_l;
      const u32x4 x = *reinterpret_cast<const AG_LDS u32x4 *>(ost + row * kRowB + ((ochunk ^ geo::key(row)) << 4));
      if (row < n_rows) __builtin_amdgcn_raw_buffer_store_b128(x, o_rsrc, orow_l * row_stride + ochunk * 16, i * RPI * row_stride, 0);
    }
  }
}


}  // namespace

// Experiment switch (environment AG_PREFILL_Q64=1, read once): the 64-queries-per-wave kernel instead of the 4-wave one.
static bool ag_prefill_q64_enabled() {
  static const bool on = [] { const char *e = getenv("AG_PREFILL_Q64"); return e && e[0] == '1'; }();
  return on;
}

// Split policy: only launches too small to hide their longest item behind other work are split; heads are
// dealt to XCDs by kept rows when there are few enough per XCD for their differences to show.
void ag_prefill_bf16_plan(int num_cu, int B, int L, int Hq, int Hkv, int D, ws_cursor &ws, ag_pf_plan *plan, float **part) {
  const int G = Hq / Hkv;
  const int GB = G >= 4 ? 4 : G;
  memset(plan, 0, sizeof(*plan));
  plan->NW = 4;  // 8 waves (one workgroup per CU, twice the queries per K/V tile) measured 4-14 % slower
  plan->BM = 32 * (plan->NW / GB);
  plan->HB = G / GB;
  plan->n_hy = B * Hkv * plan->HB;
  const int64_t items = (int64_t)((L + plan->BM - 1) / plan->BM) * plan->n_hy;
  plan->n_items = (int)items;
  plan->max_tiles = (L + kBN - 1) / kBN;
  plan->slots = (8 / plan->NW) * num_cu;
  plan->n_split = 1;
  // Two chunks at most per item, unless the items are so few (few heads) that even their halves leave workgroup
  // slots empty: then more, until the chunks cover the slots (the merge adds the states in chunk order, so it stays
  // reproducible).  Measured with 4 heads x 4096 all-kept tokens: 2 chunks 54 us, up to 4 chunks 49.5 us, up to 8
  // chunks 68 us -- the chunk that arrives last fetches the other states one after the other.
  if (items < (int64_t)8 * num_cu && plan->max_tiles > 16) {
    plan->n_split = 2;
    while (items * plan->n_split < (int64_t)plan->slots && plan->n_split < 8 && plan->max_tiles / (2 * plan->n_split) >= 8)
      plan->n_split *= 2;
  }
  *part = nullptr;
  if (plan->n_split > 1) {
    *part = ws.take<float>((size_t)items * plan->n_split * plan->NW * (D / 2 + 2) * 64);
    plan->chunk_tiles = ws.take<int32_t>(64);
    plan->tickets = ws.take<int32_t>((size_t)items);
  }
  // rows of query tiles whose items can exceed one chunk: (t + 1) BM tokens give at most that many / 64 key tiles
  const int n_qt_all = (L + plan->BM - 1) / plan->BM;
  plan->n_sp = n_qt_all;
  if (plan->n_split > 1) {
    const int lo = (plan->max_tiles + plan->n_split - 1) / plan->n_split;
    int shorter = 0;  // rows t = 0 .. shorter - 1 never exceed lo tiles
    while (shorter < n_qt_all && (std::min((shorter + 1) * plan->BM, L) + kBN - 1) / kBN <= lo) ++shorter;
    plan->n_sp = n_qt_all - shorter;
  }
  // 16 or more heads per XCD: head-major block order (K/V reuse in the L2); fewer: a head order balanced by kept rows
  plan->head_major = plan->n_split == 1 && plan->n_hy >= 128;
  if (!plan->head_major && plan->n_hy % 8 == 0 && plan->n_hy >= 16 && plan->n_hy <= 256)
    plan->order = ws.take<int32_t>(plan->n_hy);
  if (B * Hkv > 1024) {  // the planner holds the units' counts in LDS
    plan->order = nullptr;
    plan->chunk_tiles = nullptr;
    plan->n_split = 1;
    plan->tickets = nullptr;
    *part = nullptr;
  }
  if (plan->order || plan->chunk_tiles) plan->kept = ws.take<int32_t>((size_t)B * Hkv);
}

hipError_t ag_launch_prefill_bf16(hipStream_t s, const void *q, const void *k, const void *v, const uint64_t *words,
                                  const int32_t *blk_off, int B, int L, int Hq, int Hkv, int D, float qscale, int n_recent,
                                  const void *kc, const void *vc, const int64_t *row_off, void *out,
                                  const ag_pf_plan &plan, float *part, bool out_token_major, ag_evpair ev) {
  (void)B;
  const int nw = ag_nwords(L);
  const int G = Hq / Hkv;
  const int GB = G >= 4 ? 4 : G;
  if ((int64_t)plan.n_items * plan.n_split > 0x7fffffff) return hipErrorInvalidValue;
  const int n_qt = plan.n_items / plan.n_hy;
  const int64_t blocks = plan.head_major ? (int64_t)((plan.n_hy + 7) / 8) * 8 * n_qt
                                         : (int64_t)plan.n_hy * (plan.n_sp * plan.n_split + (n_qt - plan.n_sp));
  const dim3 grid((unsigned)blocks), block(64 * plan.NW);
  if (D == 128 && n_recent == 1 && ag_prefill_q64_enabled())  // 64 queries per wave: 2 waves per workgroup, same plan
    return ag_launch_prefill_d128_q64(s, q, k, v, words, blk_off, L, Hq, Hkv, qscale, kc, vc, row_off, out, plan, part,
                                      out_token_major, ev, (unsigned)blocks);
#define AG_PF(DD, GG, BB)                                                                                            \
  AG_LAUNCH(ev, (ag_prefill_bf16_kernel<DD, GG, BB, 4>), grid, block, 0, s, (const uint16_t *)q, (const uint16_t *)k,  \
            (const uint16_t *)v, words, blk_off, (const uint16_t *)kc, (const uint16_t *)vc, row_off, L, Hq, Hkv, nw,  \
            plan.n_hy, plan.n_split, plan.n_sp, plan.chunk_tiles, qscale, n_recent, plan.order, plan.head_major,        \
            (uint16_t *)out, out_token_major ? 1 : 0, part, plan.tickets)
#define AG_PFD(DD)                                                                                   \
  do {                                                                                               \
    if (n_recent > 1) {                                                                              \
      if (GB == 1) { AG_PF(DD, 1, true); } else if (GB == 2) { AG_PF(DD, 2, true); } else { AG_PF(DD, 4, true); }    \
    } else {                                                                                         \
      if (GB == 1) { AG_PF(DD, 1, false); } else if (GB == 2) { AG_PF(DD, 2, false); } else { AG_PF(DD, 4, false); } \
    }                                                                                                \
  } while (0)
  if (D == 128) AG_PFD(128); else if (D == 64) AG_PFD(64); else return hipErrorInvalidValue;
#undef AG_PFD
#undef AG_PF
  return hipGetLastError();
}
