// Gate (Eq. 3, Eq. 4): features [tokens, d_in] x W [d_in, H_f] -> logits -> keep flags.
//
// The product is a skinny GEMM (N = H_f <= 32) whose cost is reading the features once from HBM.  The bf16
// path runs it on MFMA (v_mfma_f32_32x32x16_bf16, N padded to 32): every wave owns a tile of tokens and a slice
// of the K range, fetches its feature rows as whole 128-byte lines (handed to the MFMA layout through LDS in the
// fused kernels), and takes the matching W fragments either from W as stored, transposed on the way through LDS,
// or from a pre-packed copy that stays in L2.  K is split over the waves of a workgroup.  With enough tokens one
// fused kernel does everything (ag_gate_fused_kernel; ag_norm_gate_kernel when the normalisation of the input is
// fused in as well).  With few tokens (decode-sized calls) K is also split over several workgroups of the simpler
// ag_gate_mfma_kernel; partial sums then go to the workspace and a second kernel adds them in a fixed order (so
// flags are reproducible run to run), adds the bias, compares with the logit-space threshold and writes the flags
// head-major.
#include "ag_internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
#define AG_LDS __attribute__((address_space(3)))

constexpr int kNP = 32;  // padded head count (MFMA N)

// Swizzle key of row r of a wave's 32 x 128-byte hand-over buffer: the 16-byte piece p of the row is stored at
// position p ^ xkey(r).  Rows alternate between the two halves of the 64 banks, so the 16 lanes that LDS serves
// together (2 whole rows on the writing side, 16 rows at one piece index on the reading side) need 8 different
// keys among rows of equal parity: bits 1..3 of the row.
__device__ __forceinline__ int xkey(int r) { return (r >> 1) & 7; }

// W [d_in, H_f] bf16 -> fragment order: [(chunk*4 + step)*64 + lane][8], lane = (n = lane%32, kb = lane/32),
// element j = W[chunk*64 + kb*32 + step*8 + j][n]  (0 for n >= H_f).
__global__ void ag_gate_pack_w(const uint16_t *__restrict__ w, int d_in, int H_f, uint16_t *__restrict__ wp) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;  // one packed element
  if (i >= d_in * kNP) return;
  const int j = i & 7, lane = (i >> 3) & 63, step = (i >> 9) & 3, chunk = i >> 11;
  const int n = lane & 31, kb = lane >> 5;
  const int kk = chunk * 64 + kb * 32 + step * 8 + j;
  wp[i] = n < H_f ? w[(size_t)kk * H_f + n] : (uint16_t)0;
}

// grid = (token tiles, K splits); block = 256.  partial [S][tokens_pad][32] fp32.
template <int MT>
__global__ __launch_bounds__(256) void ag_gate_mfma_kernel(const uint16_t *__restrict__ x, const uint4 *__restrict__ wp,
                                                           int64_t tokens, int d_in, int chunks_per_split,
                                                           float *__restrict__ partial, int64_t tokens_pad) {
  __shared__ float red[4][MT][32][33];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 31, kb = lane >> 5;
  const int64_t tok0 = (int64_t)blockIdx.x * (32 * MT);
  const int nchunks = d_in / 64;
  const int c_begin = blockIdx.y * chunks_per_split;
  const int c_end = min(nchunks, c_begin + chunks_per_split);

  const uint4 *rows[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    int64_t tok = tok0 + t * 32 + m;
    if (tok >= tokens) tok = tokens - 1;  // clamp: the row is read but its result is never written
    rows[t] = reinterpret_cast<const uint4 *>(x + (size_t)tok * d_in + kb * 32);
  }
  f32x16 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  for (int c = c_begin + wave; c < c_end; c += 4) {
    uint4 a[MT][4], b[4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int s = 0; s < 4; ++s) a[t][s] = rows[t][c * 8 + s];  // 64 k = 8 uint4 per row; this lane's half
#pragma unroll
    for (int s = 0; s < 4; ++s) b[s] = wp[((size_t)c * 4 + s) * 64 + lane];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int t = 0; t < MT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[t][s]),
                                                         __builtin_bit_cast(bf16x8, b[s]), acc[t], 0, 0, 0);
  }
  // C layout of the 32x32 tile: acc[r] is (row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32)
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][t][8 * (r >> 2) + 4 * kb + (r & 3)][m] = acc[t][r];
  __syncthreads();
  float *dst = partial + ((size_t)blockIdx.y * tokens_pad + tok0) * kNP;
  for (int e = threadIdx.x; e < MT * 32 * 32; e += 256) {
    const int t = e >> 10, row = (e >> 5) & 31, col = e & 31;
    dst[e] = red[0][t][row][col] + red[1][t][row][col] + red[2][t][row][col] + red[3][t][row][col];
  }
}

// One workgroup of 8 waves per tile of TOK = 32 or 16 tokens and K split (grid.y splits; wave w takes 64-wide
// chunks w, w + 8, ... of its split, PF of them in flight), the 8 partial tiles added in wave order through LDS.
// (TOK = 16: launches with fewer 32-token tiles than CUs; the upper half of the MFMA then repeats the lower.)  With one split the workgroup
// goes on to bias, threshold, logits and head-major flags.  With several, each stores its 32x32 partial tile
// (written through the caches, complete before its arrival is counted) and the split that arrives last adds all
// of them in split order -- the same order whoever is last, so the flags are reproducible -- and finishes.
// The arrival counters live in the context, start at zero and are set back to zero by the split that arrives
// last, so no launch has to clear them.
//
// RAW: W is taken as the caller stores it ([d_in, H_f] row-major, H_f a multiple of 4, 16-byte aligned).  A wave
// copies the 64 rows of a chunk into its own 4 KiB of LDS and reads them back with the transposing LDS read,
// which hands lane (n, kb) the eight rows kb*32 + step*8 + 0..7 of column n: the B operand that matches the
// A operand (lane = token m and half kb: features kb*32 + step*8 + 0..7).  Columns n >= H_f read whatever follows in LDS; they only reach output
// columns that are never stored.  Otherwise wp holds the fragments prepared by ag_gate_pack_w.
constexpr int kFusedWaves = 8;
template <bool RAW, int PF, int TOK>
__global__ __launch_bounds__(64 * kFusedWaves, PF == 2 ? 2 : 1) void ag_gate_fused_kernel(
    const uint16_t *__restrict__ x, const uint4 *__restrict__ wp, int64_t tokens, int d_in, int L, int H_f,
    const float *__restrict__ bias, float thr, int n_sink, float *__restrict__ logits, uint8_t *__restrict__ flags,
    float *__restrict__ partial, int32_t *__restrict__ tickets) {
  // [wave][4 KiB]: W staging of the wave while it accumulates, afterwards its 32 x 32 fp32 partial tile
  __shared__ __attribute__((aligned(16))) uint8_t wst[kFusedWaves][4096];
  // [wave][4 KiB]: a chunk of the wave's 32 feature rows on its way from the memory-side layout to the A layout
  __shared__ __attribute__((aligned(16))) uint8_t xstage[kFusedWaves][4096];
  __shared__ uint8_t fl[kNP][32];
  __shared__ int is_last;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: chunk offsets stay in SGPRs
  const int m = lane & 31, kb = lane >> 5;
  const int ma = m & (TOK - 1);  // A row this lane reads: with 16-token tiles the upper half of the MFMA repeats the lower
  const int lr = lane >> 3, lp = lane & 7;  // row within a group of 8 and 16-byte piece of the memory-side layout
  constexpr int NI = TOK / 8;  // load instructions per chunk: 8 rows each
  const int64_t tok0 = (int64_t)blockIdx.x * TOK;
  const int nchunks = d_in / 64;
  const int splits = gridDim.y, split = blockIdx.y;
  const int c_lo = (int)((int64_t)nchunks * split / splits), c_hi = (int)((int64_t)nchunks * (split + 1) / splits);
  // Feature rows: a chunk (64 features) is one 128-byte line per row, and a load instruction fetches 8 whole
  // lines (lane -> row 8 i + lane / 8, 16-byte piece lane % 8) instead of 64 scattered 16-byte pieces, which the
  // texture path would take four times as long to address.  Rows past the last token repeat the last row (read,
  // never written).  The chunk then goes through the wave's LDS buffer (pieces XOR-swizzled with the row, so that
  // neither side has bank conflicts) to the A layout: lane (token m, half kb), step s: features kb*32 + s*8 .. +7.
  const int rows = (int)min((int64_t)TOK, tokens - tok0);
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(x + (size_t)tok0 * d_in), 0, (uint32_t)rows * (uint32_t)d_in * 2u, 0x00020000);
  int row_off[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) row_off[i] = min(8 * i + lr, rows - 1) * d_in * 2 + lp * 16;
  AG_LDS uint8_t *xst = (AG_LDS uint8_t *)xstage[wave];
  // RAW: a chunk is 64 * H_f * 2 bytes = 8 * H_f uint4, lane l holds uint4 l, l + 64, ... of it
  const int chunk_u4 = 8 * H_f;
  AG_LDS uint8_t *stage = (AG_LDS uint8_t *)wst[wave];
  // transposing read: the 16 lanes of a group give the addresses of 4 rows x 16 columns (lane i: row i / 4,
  // columns 4 (i % 4) ..+3) and lane i receives column i of the 4 rows
  const int gl = lane >> 4, li = lane & 15;
  const int tr_col = min(16 * (gl & 1) + 4 * (li & 3), H_f - 4);
  const int tr_off = ((gl >> 1) * 32 + (li >> 2)) * (H_f * 2) + tr_col * 2;
  auto wave_sync = [] {  // lanes of one wave exchange data through LDS
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int c0 = c_lo + wave; c0 < c_hi; c0 += kFusedWaves * PF) {
    uint4 a[PF][4], b[PF][4];
    // W first: its loads hit the L2 and return early, so the staging below runs while the feature rows are
    // still on their way from HBM (a wave's loads return in issue order)
#pragma unroll
    for (int p = 0; p < PF; ++p) {
      const int c = min(c0 + kFusedWaves * p, c_hi - 1);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (RAW) {
          const int i = min(s * 64 + lane, chunk_u4 - 1);
          b[p][s] = wp[(size_t)c * chunk_u4 + i];
        } else {
          b[p][s] = wp[((size_t)c * 4 + s) * 64 + lane];
        }
      }
    }
#pragma unroll
    for (int p = 0; p < PF; ++p) {
      const int c = min(c0 + kFusedWaves * p, c_hi - 1);
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, row_off[i], c * 128, 0);
        a[p][i] = make_uint4(t[0], t[1], t[2], t[3]);
      }
    }
    if (RAW) {
#pragma unroll
      for (int p = 0; p < PF; ++p) {
        wave_sync();  // the fragments of the previous chunk have been read
#pragma unroll
        for (int s = 0; s < 4; ++s)
          if (s * 64 + lane < chunk_u4)
            *reinterpret_cast<AG_LDS u32x4 *>(stage + (s * 64 + lane) * 16) =
                u32x4{b[p][s].x, b[p][s].y, b[p][s].z, b[p][s].w};
        wave_sync();  // the chunk's rows are there for every lane
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(stage + tr_off + (s * 8) * (H_f * 2)));
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(stage + tr_off + (s * 8 + 4) * (H_f * 2)));
          b[p][s] = __builtin_bit_cast(uint4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
      }
    }
#pragma unroll
    for (int p = 0; p < PF; ++p)
      if (c0 + kFusedWaves * p < c_hi) {
        wave_sync();  // the previous chunk's fragments have been read
#pragma unroll
        for (int i = 0; i < NI; ++i)
          *reinterpret_cast<AG_LDS u32x4 *>(xst + (8 * i + lr) * 128 + ((lp ^ xkey(8 * i + lr)) << 4)) =
              u32x4{a[p][i].x, a[p][i].y, a[p][i].z, a[p][i].w};
        wave_sync();  // the chunk's rows are there for every lane
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const u32x4 t = *reinterpret_cast<const AG_LDS u32x4 *>(xst + ma * 128 + (((kb * 4 + s) ^ xkey(ma)) << 4));
          a[p][s] = make_uint4(t[0], t[1], t[2], t[3]);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[p][s]),
                                                        __builtin_bit_cast(bf16x8, b[p][s]), acc, 0, 0, 0);
      }
  }
  float(*red)[32][32] = reinterpret_cast<float(*)[32][32]>(wst);
  if (RAW) wave_sync();  // the wave's staging area becomes its partial tile
#pragma unroll
  for (int r = 0; r < 16; ++r) red[wave][8 * (r >> 2) + 4 * kb + (r & 3)][m] = acc[r];
  __syncthreads();
  // element e = (token row e / 32, head e % 32); thread t owns e = t and t + 512
  float v[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = threadIdx.x + 64 * kFusedWaves * i;
    v[i] = 0.f;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) v[i] += red[w][e >> 5][e & 31];
  }
  if (splits > 1) {
    float *tile = partial + (size_t)blockIdx.x * splits * 1024;
#pragma unroll
    for (int i = 0; i < 2; ++i)
      __hip_atomic_store(&tile[split * 1024 + threadIdx.x + 64 * kFusedWaves * i], v[i], __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_SYSTEM);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
      is_last = __hip_atomic_fetch_add(&tickets[blockIdx.x], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == splits - 1;
    __syncthreads();
    if (!is_last) return;
    if (threadIdx.x == 0) tickets[blockIdx.x] = 0;  // ready for the next launch
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float sum = 0.f;
      for (int sp = 0; sp < splits; ++sp) {
        const float other = __hip_atomic_load(&tile[sp * 1024 + threadIdx.x + 64 * kFusedWaves * i], __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_SYSTEM);
        sum += sp == split ? v[i] : other;
      }
      v[i] = sum;
    }
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = threadIdx.x + 64 * kFusedWaves * i;
    const int rw = e >> 5, h = e & 31;
    const int64_t tk = tok0 + rw;
    if (h < H_f && rw < TOK && tk < tokens) {
      const float val = v[i] + bias[h];
      if (logits) logits[(size_t)tk * H_f + h] = val;
      fl[h][rw] = (val > thr || (int)(tk % L) < n_sink) ? 1 : 0;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 32 * H_f; e += 64 * kFusedWaves) {
    const int h = e >> 5, rw = e & 31;
    const int64_t tk = tok0 + rw;
    if (rw >= TOK || tk >= tokens) continue;
    const int64_t b = tk / L;
    flags[((size_t)b * H_f + h) * L + (tk - b * L)] = fl[h][rw];
  }
}

// RMS normalisation fused with the gate: x = h / sqrt(mean_c h^2 + eps) * g, rounded once to bf16, written out for
// the projections that follow, and multiplied by W from the same registers, so the gate costs no second read of x.
// One workgroup of 8 waves per 32 tokens.  Wave w owns the 64-feature chunks w, w + 8, ... (at most NCH of
// them: d_in <= 4096 with 32-token tiles, <= 8192 with 16-token tiles) of all rows of the tile and keeps them in registers for the whole kernel, so all loads of the tile are
// in flight at once.  A chunk is one 128-byte line per row; a load or store instruction moves 8 whole lines (lane
// -> row 8 i + lane / 8, 16-byte piece lane % 8).  The squares are summed per lane, over the 8 lanes of a row and
// then over the waves through LDS in wave order.  After the scaling the chunk is stored from the same registers
// and handed through a 4 KiB LDS buffer of the wave (pieces XOR-swizzled with the row: no bank conflicts on either
// side) to the MFMA's A layout, lane (token m, half kb) holding features kb*32 + s*8 .. +7 for step s.  That
// layout, the W fragments and the order of the MFMAs (chunks ascending per wave, then the waves in order) are
// those of ag_gate_fused_kernel with one K split, so the logits are those ag_gate gives on the stored x bit for
// bit whenever that kernel runs unsplit.
template <bool RAW, int TOK, int NCH>  // NCH = chunks a wave holds: d_in <= 8 waves x NCH x 64 features
__global__ __launch_bounds__(64 * kFusedWaves, TOK == 16 ? 2 : 1) void ag_norm_gate_kernel(
    const uint16_t *h, const uint16_t *__restrict__ g, float eps, const uint4 *__restrict__ wp,
    int64_t tokens, int d_in, int L, int H_f, const float *__restrict__ bias, float thr, int n_sink,
    uint16_t *x_out, float *__restrict__ logits, uint8_t *__restrict__ flags) {
  // [wave][4 KiB]: the wave's hand-over buffer (chunk of x, then chunk of W), afterwards its 32 x 32 fp32 partial tile
  __shared__ __attribute__((aligned(16))) uint8_t wst[kFusedWaves][2][4096];
  __shared__ __attribute__((aligned(16))) uint16_t g_l[kFusedWaves * NCH * 64];
  __shared__ float ssq_l[kFusedWaves][32];
  __shared__ uint8_t fl[kNP][32];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: chunk offsets stay in SGPRs
  constexpr int NI = TOK / 8;  // load / store instructions per chunk: 8 rows each
  const int m = lane & 31, kb = lane >> 5;
  const int ma = m & (TOK - 1);  // A row this lane reads: with 16-token tiles the upper half of the MFMA repeats the lower
  const int lr = lane >> 3, lp = lane & 7;  // row within a group of 8 and 16-byte piece of the memory-side layout
  const int64_t tok0 = (int64_t)blockIdx.x * TOK;
  const int nchunks = d_in / 64;
  // The tile's rows through buffer descriptors: a load or store is one per-lane offset plus a scalar chunk offset.
  // Rows past the last token are read as the last token's row again and never stored.
  const int rows = (int)min((int64_t)TOK, tokens - tok0);
  const uint32_t tile_bytes = (uint32_t)rows * (uint32_t)d_in * 2u;
  const __amdgpu_buffer_rsrc_t h_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(h + (size_t)tok0 * d_in), 0, tile_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(x_out + (size_t)tok0 * d_in), 0, tile_bytes, 0x00020000);
  int row_off[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) row_off[i] = min(8 * i + lr, rows - 1) * d_in * 2 + lp * 16;
  auto to_u4 = [](u32x4 v) { return make_uint4(v[0], v[1], v[2], v[3]); };
  uint4 a[NCH][NI];
#pragma unroll
  for (int p = 0; p < NCH; ++p) {
    const int c = min(wave + kFusedWaves * p, nchunks - 1);
#pragma unroll
    for (int i = 0; i < NI; ++i) a[p][i] = to_u4(__builtin_amdgcn_raw_buffer_load_b128(h_rsrc, row_off[i], c * 128, 0));
  }
  // W fragments (see ag_gate_fused_kernel for the two forms of wp), requested two chunks ahead of their use
  const int chunk_u4 = 8 * H_f;
  const __amdgpu_buffer_rsrc_t w_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)wp, 0, (uint32_t)d_in * (RAW ? H_f : kNP) * 2u, 0x00020000);
  int w_off[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) w_off[s] = RAW ? min(s * 64 + lane, chunk_u4 - 1) * 16 : s * 1024 + lane * 16;
  auto load_w = [&](uint4 (&bw)[4], int p) {
    const int c = min(wave + kFusedWaves * p, nchunks - 1);
#pragma unroll
    for (int s = 0; s < 4; ++s)
      bw[s] = to_u4(__builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_off[s], c * (RAW ? chunk_u4 * 16 : 4096), 0));
  };
  uint4 b[3][4];
  load_w(b[0], 0);
  load_w(b[1], 1);
  // the normalisation weights: 16 bytes per thread and round cover 4096 of them
  for (int i = (int)threadIdx.x * 8; i < d_in; i += 64 * kFusedWaves * 8)
    *reinterpret_cast<uint4 *>(&g_l[i]) = *reinterpret_cast<const uint4 *>(g + i);

  float ssq[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) ssq[i] = 0.f;
#pragma unroll
  for (int p = 0; p < NCH; ++p)
    if (wave + kFusedWaves * p < nchunks) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const uint32_t wd[4] = {a[p][i].x, a[p][i].y, a[p][i].z, a[p][i].w};
        // two squares per instruction, on the packed pair as it is (v_dot2_f32_bf16, fp32 sum)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          ssq[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, wd[e]), __builtin_bit_cast(bf16x2, wd[e]), ssq[i], false);
      }
    }
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    ssq[i] += __shfl_xor(ssq[i], 1, 64);
    ssq[i] += __shfl_xor(ssq[i], 2, 64);
    ssq[i] += __shfl_xor(ssq[i], 4, 64);
    if (lp == 0) ssq_l[wave][8 * i + lr] = ssq[i];
  }
  __syncthreads();  // (also publishes g_l)
  float r[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) tot += ssq_l[w][8 * i + lr];
    r[i] = 1.f / sqrtf(tot / (float)d_in + eps);
  }

  AG_LDS uint8_t *xst = (AG_LDS uint8_t *)wst[wave][0], *stage = (AG_LDS uint8_t *)wst[wave][1];
  const int gl = lane >> 4, li = lane & 15;
  const int tr_col = min(16 * (gl & 1) + 4 * (li & 3), H_f - 4);
  const int tr_off = ((gl >> 1) * 32 + (li >> 2)) * (H_f * 2) + tr_col * 2;
  auto wave_sync = [] {  // lanes of one wave exchange data through LDS
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  f32x16 acc;
#pragma unroll
  for (int r16 = 0; r16 < 16; ++r16) acc[r16] = 0.f;
#pragma unroll
  for (int p = 0; p < NCH; ++p) {
    __builtin_amdgcn_sched_barrier(0);  // one chunk at a time: interleaving them costs more registers than it hides
    if (p + 2 < NCH) load_w(b[(p + 2) % 3], p + 2);
    const bool valid = wave + kFusedWaves * p < nchunks;  // wave-uniform
    const int c = wave + kFusedWaves * p;
    if (valid) {
      const uint4 gw = *reinterpret_cast<const uint4 *>(&g_l[c * 64 + lp * 8]);
      const uint32_t gd[4] = {gw.x, gw.y, gw.z, gw.w};
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const uint32_t hd[4] = {a[p][i].x, a[p][i].y, a[p][i].z, a[p][i].w};
        uint32_t xd[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = (__uint_as_float(hd[e] << 16) * r[i]) * __uint_as_float(gd[e] << 16);
          const float hi = (__uint_as_float(hd[e] & 0xffff0000u) * r[i]) * __uint_as_float(gd[e] & 0xffff0000u);
          const f32x2 pr = {lo, hi};
          xd[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
        }
        const u32x4 xv = {xd[0], xd[1], xd[2], xd[3]};
        if (8 * i + lr < rows) __builtin_amdgcn_raw_buffer_store_b128(xv, x_rsrc, row_off[i], c * 128, 0);
        *reinterpret_cast<AG_LDS u32x4 *>(xst + (8 * i + lr) * 128 + ((lp ^ xkey(8 * i + lr)) << 4)) = xv;
      }
    }
    uint4(&bw)[4] = b[p % 3];
    if (RAW) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (s * 64 + lane < chunk_u4)
          *reinterpret_cast<AG_LDS u32x4 *>(stage + (s * 64 + lane) * 16) = u32x4{bw[s].x, bw[s].y, bw[s].z, bw[s].w};
    }
    wave_sync();  // the chunk's x rows and W rows are there for every lane
    if (RAW) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(stage + tr_off + (s * 8) * (H_f * 2)));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(stage + tr_off + (s * 8 + 4) * (H_f * 2)));
        bw[s] = __builtin_bit_cast(uint4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
    }
    if (valid) {
      u32x4 af[4];
#pragma unroll
      for (int s = 0; s < 4; ++s)
        af[s] = *reinterpret_cast<const AG_LDS u32x4 *>(xst + ma * 128 + (((kb * 4 + s) ^ xkey(ma)) << 4));
#pragma unroll
      for (int s = 0; s < 4; ++s)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[s]),
                                                      __builtin_bit_cast(bf16x8, bw[s]), acc, 0, 0, 0);
    }
    wave_sync();  // both buffers have been read
  }
  float(*red)[32][32] = reinterpret_cast<float(*)[32][32]>(wst);
  __syncthreads();  // (red[w] is not wave w's own buffer)
#pragma unroll
  for (int r16 = 0; r16 < 16; ++r16) red[wave][8 * (r16 >> 2) + 4 * kb + (r16 & 3)][m] = acc[r16];
  __syncthreads();
  // element e = (token row e / 32, head e % 32); thread t owns e = t and t + 512
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = threadIdx.x + 64 * kFusedWaves * i;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) v += red[w][e >> 5][e & 31];
    const int rw = e >> 5, hh = e & 31;
    const int64_t tk = tok0 + rw;
    if (hh < H_f && rw < TOK && tk < tokens) {
      const float val = v + bias[hh];
      if (logits) logits[(size_t)tk * H_f + hh] = val;
      fl[hh][rw] = (val > thr || (int)(tk % L) < n_sink) ? 1 : 0;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 32 * H_f; e += 64 * kFusedWaves) {
    const int hh = e >> 5, rw = e & 31;
    const int64_t tk = tok0 + rw;
    if (rw >= TOK || tk >= tokens) continue;
    const int64_t bb = tk / L;
    flags[((size_t)bb * H_f + hh) * L + (tk - bb * L)] = fl[hh][rw];
  }
}

// fp32 features: plain ALU path (one thread per (token, padded head)), partial [1][tokens_pad][32].
__global__ __launch_bounds__(256) void ag_gate_f32_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                          int64_t tokens, int d_in, int H_f,
                                                          float *__restrict__ partial) {
  const int h = threadIdx.x & 31;
  const int64_t tok = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
  if (tok >= tokens) return;
  float s = 0.f;
  if (h < H_f) {
    const float *xr = x + (size_t)tok * d_in;
    for (int c = 0; c < d_in; ++c) s = fmaf(xr[c], w[(size_t)c * H_f + h], s);
  }
  partial[(size_t)tok * kNP + h] = s;
}

// Sum the K splits in order, add bias, threshold, write logits [tokens, H_f] and flags [B, H_f, L].
constexpr int kFinTok = 16;  // tokens per finalize workgroup

__global__ __launch_bounds__(256) void ag_gate_finalize_kernel(const float *__restrict__ partial, int splits,
                                                               int64_t tokens_pad, int64_t tokens, int L, int H_f,
                                                               const float *__restrict__ bias, float thr, int n_sink,
                                                               float *__restrict__ logits,
                                                               uint8_t *__restrict__ flags) {
  __shared__ uint8_t fl[kNP][kFinTok];
  const int64_t tok0 = (int64_t)blockIdx.x * kFinTok;
  const int h = threadIdx.x & 31;
  // thread -> (token tok0 + tid/32 [+ 8], head h): the K splits of both elements are fetched as independent loads
  float s[2] = {0.f, 0.f};
  int64_t tok[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) tok[i] = min(tok0 + (threadIdx.x >> 5) + 8 * i, tokens - 1);
#pragma unroll 4
  for (int sp = 0; sp < splits; ++sp)
#pragma unroll
    for (int i = 0; i < 2; ++i) s[i] += partial[((size_t)sp * tokens_pad + tok[i]) * kNP + h];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int tl = (threadIdx.x >> 5) + 8 * i;
    if (h < H_f && tok0 + tl < tokens) {
      const float v = s[i] + bias[h];
      if (logits) logits[(size_t)tok[i] * H_f + h] = v;
      const int t = (int)(tok[i] % L);
      fl[h][tl] = (v > thr || t < n_sink) ? 1 : 0;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < kFinTok * H_f; e += 256) {
    const int hh = e / kFinTok, tl = e - hh * kFinTok;
    const int64_t tk = tok0 + tl;
    if (tk >= tokens) continue;
    const int64_t b = tk / L;
    const int t = (int)(tk - b * L);
    flags[((size_t)b * H_f + hh) * L + t] = fl[hh][tl];
  }
}

struct gate_plan {
  int mt, tiles, splits, chunks_per_split;
  int64_t tokens_pad;
};

gate_plan plan_gate(int64_t tokens, int d_in, ag_dtype dt, int num_cu) {
  gate_plan p;
  if (dt != AG_BF16) {
    p.mt = 1; p.tiles = (int)((tokens + 7) / 8); p.splits = 1; p.chunks_per_split = 0;
    p.tokens_pad = (tokens + 63) / 64 * 64;
    return p;
  }
  const int nchunks = d_in / 64;
  p.mt = tokens >= (int64_t)64 * 8 * num_cu ? 2 : 1;
  p.tiles = (int)((tokens + 32 * p.mt - 1) / (32 * p.mt));
  // enough workgroups to cover the chip about 4 times, but at least 4 chunks (one per wave) per split
  int want = (4 * num_cu + p.tiles - 1) / p.tiles;
  int max_splits = nchunks / 4 > 0 ? nchunks / 4 : 1;
  p.splits = want < 1 ? 1 : (want > max_splits ? max_splits : want);
  if (p.splits > 16) p.splits = 16;
  p.chunks_per_split = (nchunks + p.splits - 1) / p.splits;
  p.splits = (nchunks + p.chunks_per_split - 1) / p.chunks_per_split;
  p.tokens_pad = (int64_t)p.tiles * 32 * p.mt;
  if (p.tokens_pad % 64) p.tokens_pad += 32;
  return p;
}

}  // namespace

size_t ag_ws_gate_bytes(int64_t tokens, int d_in, int H_f, ag_dtype dt) {
  (void)H_f;
  // worst case over the plans plan_gate can pick (num_cu is not known here): 16 splits
  const int64_t tokens_pad = (tokens + 63) / 64 * 64;
  const size_t part = ag_align256((size_t)16 * tokens_pad * kNP * sizeof(float));
  const size_t pack = dt == AG_BF16 ? ag_align256((size_t)d_in * kNP * 2) : 0;
  return part + pack;
}

hipError_t ag_launch_gate(ag_ctx *ctx, hipStream_t s, const void *feat, ag_dtype dt, int B, int L, int d_in,
                          const void *w, const float *bias, int H_f, float thr, int n_sink, float *logits,
                          uint8_t *flags, ws_cursor &ws) {
  const int64_t tokens = (int64_t)B * L;
  const gate_plan p = plan_gate(tokens, d_in, dt, ctx->num_cu);
  const int64_t tiles32 = (tokens + 31) / 32;
  const bool fused = dt == AG_BF16 && tiles32 >= ctx->num_cu / 4;  // enough token tiles: one fused kernel
  // the fused kernel reads W as stored when its rows can be moved and transposed in 8- and 16-byte pieces
  const bool raw_w = fused && H_f % 4 == 0 && (reinterpret_cast<uintptr_t>(w) & 15) == 0;
  // Fewer 32-token tiles than CUs: tiles of 16 tokens first (twice the workgroups, no exchange of partial sums
  // between them; the MFMA's upper half then idles, which costs nothing here), K splits only after that.
  const bool tok16 = raw_w && tiles32 < ctx->num_cu;
  const int64_t tiles = tok16 ? (tokens + 15) / 16 : tiles32;
  int fsplits = 1;
  if (fused) {  // K splits until the chip is covered, each wave keeping at least 2 chunks
    while (tiles * fsplits < ctx->num_cu && d_in / 64 / (fsplits * 2) >= 2 * kFusedWaves && fsplits < 8 &&
           tiles <= kGateTickets)
      fsplits *= 2;
  }
  float *partial = fused ? (fsplits > 1 ? ws.take<float>((size_t)tiles * fsplits * 1024) : nullptr)
                         : ws.take<float>((size_t)p.splits * p.tokens_pad * kNP);
  int32_t *tickets = fused && fsplits > 1 ? ctx->gate_tickets : nullptr;
  uint16_t *wp = dt == AG_BF16 && !raw_w ? ws.take<uint16_t>((size_t)d_in * kNP) : nullptr;
  if (!ws.ok) return hipSuccess;  // caller reports AG_EWORKSPACE
  if (dt == AG_BF16) {
    if (!raw_w) {
      const int n = d_in * kNP;
      hipLaunchKernelGGL(ag_gate_pack_w, dim3((n + 255) / 256), dim3(256), 0, s, (const uint16_t *)w, d_in, H_f, wp);
    }
    if (fused) {
      const dim3 grid((unsigned)tiles, fsplits), block(64 * kFusedWaves);
      const ag_evpair ev = ag_time_kernel(ctx, AG_K_GATE);
      // PF = feature chunks a wave keeps in flight.  A launch of at most one workgroup per CU is one round of loads
      // per wave (PF = 4); a longer one runs two workgroups per CU with half the registers (PF = 2), so that one
      // loads while the other reduces and writes its flags.
      const bool two_per_cu = (int64_t)tiles * fsplits > ctx->num_cu;
#define AG_GATE_FUSED(RAWV, PFV, WPTR) AG_GATE_FUSED_T(RAWV, PFV, 32, WPTR)
#define AG_GATE_FUSED_T(RAWV, PFV, TOKV, WPTR)                                                                            \
  AG_LAUNCH(ev, (ag_gate_fused_kernel<RAWV, PFV, TOKV>), grid, block, 0, s, (const uint16_t *)feat, (const uint4 *)(WPTR), \
                     tokens, d_in, L, H_f, bias, thr, n_sink, logits, flags, partial, tickets)
      if (tok16) {  // (16-token tiles hold half the bytes per chunk: 8 chunks in flight when a wave has that many)
        if (d_in / 64 / fsplits > 4 * kFusedWaves) AG_GATE_FUSED_T(true, 8, 16, w); else AG_GATE_FUSED_T(true, 4, 16, w);
      } else if (raw_w) {
        if (two_per_cu) AG_GATE_FUSED(true, 2, w); else AG_GATE_FUSED(true, 4, w);
      } else {
        AG_GATE_FUSED(false, 4, wp);  // measured: the pre-packed path is slower with two workgroups per CU
      }
#undef AG_GATE_FUSED
#undef AG_GATE_FUSED_T
      return hipGetLastError();
    }
    const dim3 grid(p.tiles, p.splits);
    ag_tick(ctx, AG_K_GATE, s);
    if (p.mt == 2)
      hipLaunchKernelGGL(ag_gate_mfma_kernel<2>, grid, dim3(256), 0, s, (const uint16_t *)feat, (const uint4 *)wp,
                         tokens, d_in, p.chunks_per_split, partial, p.tokens_pad);
    else
      hipLaunchKernelGGL(ag_gate_mfma_kernel<1>, grid, dim3(256), 0, s, (const uint16_t *)feat, (const uint4 *)wp,
                         tokens, d_in, p.chunks_per_split, partial, p.tokens_pad);
    ag_tock(ctx, AG_K_GATE, s);
  } else {
    ag_tick(ctx, AG_K_GATE, s);
    hipLaunchKernelGGL(ag_gate_f32_kernel, dim3(p.tiles), dim3(256), 0, s, (const float *)feat, (const float *)w,
                       tokens, d_in, H_f, partial);
    ag_tock(ctx, AG_K_GATE, s);
  }
  ag_tick(ctx, AG_K_GATE_FINALIZE, s);
  hipLaunchKernelGGL(ag_gate_finalize_kernel, dim3((unsigned)((tokens + kFinTok - 1) / kFinTok)), dim3(256), 0, s, partial,
                     p.splits, p.tokens_pad, tokens, L, H_f, bias, thr, n_sink, logits, flags);
  ag_tock(ctx, AG_K_GATE_FINALIZE, s);
  return hipGetLastError();
}

hipError_t ag_launch_norm_gate(ag_ctx *ctx, hipStream_t s, const void *h, int B, int L, int d_in, const void *g,
                               float eps, const void *w, const float *bias, int H_f, float thr, int n_sink,
                               void *x_out, float *logits, uint8_t *flags, ws_cursor &ws) {
  const int64_t tokens = (int64_t)B * L;
  const bool raw_w = H_f % 4 == 0 && (reinterpret_cast<uintptr_t>(w) & 15) == 0;
  uint16_t *wp = raw_w ? nullptr : ws.take<uint16_t>((size_t)d_in * kNP);
  if (!ws.ok) return hipSuccess;  // caller reports AG_EWORKSPACE
  if (!raw_w) {
    const int n = d_in * kNP;
    hipLaunchKernelGGL(ag_gate_pack_w, dim3((n + 255) / 256), dim3(256), 0, s, (const uint16_t *)w, d_in, H_f, wp);
  }
  // tiles of 16 tokens while 32-token tiles would leave CUs without a workgroup (measured at 4096 features: 4096
  // tokens 17.8 us against 22.0 us; from 8192 tokens on the 32-token tiles are 5-10 % faster); rows of more than
  // 4096 features always take them, with 16 chunks per wave (the same registers as 32 tokens x 8 chunks)
  const bool wide = d_in > 4096;
  const bool tok16 = wide || (tokens + 31) / 32 < ctx->num_cu;
  const dim3 grid((unsigned)((tokens + (tok16 ? 15 : 31)) / (tok16 ? 16 : 32))), block(64 * kFusedWaves);
  const ag_evpair ev = ag_time_kernel(ctx, AG_K_NORM_GATE);
#define AG_NORM_GATE(RAWV, TOKV, NCHV, WPTR)                                                                              \
  AG_LAUNCH(ev, (ag_norm_gate_kernel<RAWV, TOKV, NCHV>), grid, block, 0, s, (const uint16_t *)h, (const uint16_t *)g, eps, \
            (const uint4 *)(WPTR), tokens, d_in, L, H_f, bias, thr, n_sink, (uint16_t *)x_out, logits, flags)
  if (raw_w) {
    if (wide) AG_NORM_GATE(true, 16, 16, w); else if (tok16) AG_NORM_GATE(true, 16, 8, w); else AG_NORM_GATE(true, 32, 8, w);
  } else {
    if (wide) AG_NORM_GATE(false, 16, 16, wp); else if (tok16) AG_NORM_GATE(false, 16, 8, wp); else AG_NORM_GATE(false, 32, 8, wp);
  }
#undef AG_NORM_GATE
  return hipGetLastError();
}
