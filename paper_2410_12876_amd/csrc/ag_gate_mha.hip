// The paper's main Attention-Gate module (Sec. 3.3, Eq. 3): a small multi-head attention MHA' in front of the
// gate's output projection,
//     Q', K', V' = X W'        (d -> h' heads of d'_k each)
//     A          = causal softmax attention per head over the whole prompt (no eviction inside the gate)
//     logits     = concat_heads(A) W^{O'} + bias     -> flags as in ag_gate (Eq. 4)
// Three stages, all bf16 with fp32 accumulation, d'_k = 128:
//   1. ag_proj_gemm_kernel: X [tokens, d] . W_qkv [d, 3 h' 128] on v_mfma_f32_32x32x16_bf16, written head-major
//      ([3][B, h', L, 128]) so that stage 2 reads it like any Q/K/V.
//   2. the tuned D = 128 prefill kernel with every flag set: the "compacted" rows of a head are then its K'/V'
//      themselves, so no copy is made; the output is written token-major [B, L, h' 128], the feature layout of
//   3. the gate kernels of ag_gate.hip with d_in = h' 128 and W_g = W^{O'}.
#include <string.h>

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

constexpr int kDh = 128;           // d'_k
constexpr int kBM = 128;           // tokens per workgroup tile
constexpr int kBNc = 128;          // output columns per workgroup tile
constexpr int kBK = 64;            // k per pipeline step
constexpr int kXRowB = kBK * 2;    // bytes per row of the X tile in LDS (128)
constexpr int kWRowB = kBNc * 2;   // bytes per row of the W tile in LDS (256)
constexpr int kXTileB = kBM * kXRowB;  // 16 KiB
constexpr int kWTileB = kBK * kWRowB;  // 16 KiB

__device__ __forceinline__ int swz_w(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }  // 16 chunks per W row
__device__ __forceinline__ int swz_x(int r) { return (r >> 1) & 7; }                     // 8 chunks per X row

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  const f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// C^T[n, m] = sum_k W[k, n] X[m, k]: the A operand is W^T (transposing LDS reads of the row-major W tile), the B
// operand is X^T (16-byte LDS reads of the row-major X tile), so a lane ends up with 4 consecutive output columns
// of one token -- 8-byte stores into the head-major result.
//   x [M, K] bf16 row-major, w [K, N] bf16 row-major, K % 64 == 0, N % 128 == 0, N = 3 * hp * 128.
//   out: three tensors [B, hp, L, 128] back to back; token m = b * L + t.
// grid = (N / 128, ceil(M / 128)); 4 waves, wave (wn, wm) owns the 64 x 64 quadrant of the tile.
//
// COMPACT (the layer's own K/V projection, N = 2 * hp * 128: K columns, then V columns): besides the two full tensors
// -- every token needs its own k, v for the diagonal of Eq. 5 -- a tile, which is 128 tokens of one head, also
// writes the rows of its kept tokens straight into the ragged cache, at the position the flag scan gives them
// (words / blk_off: 64-bit keep masks and their exclusive prefix counts), so the compaction pass and its re-read of
// K and V disappear.  The K tiles also write idx, the first token tile of a K head writes len.
struct ag_proj_compact {
  const uint64_t *words;    // [units, nw]
  const int32_t *blk_off;   // [units, nw + 1]
  const int64_t *row_off;   // [units + 1]
  uint16_t *kc, *vc;        // cache rows
  int32_t *idx, *len, *d_err;
  int nw, pos0;
};

template <bool COMPACT>
__global__ __launch_bounds__(256, 2) void ag_proj_gemm_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w,
                                                              int64_t M, int K, int N, int L, int hp,
                                                              uint16_t *__restrict__ out, ag_proj_compact cp) {
  __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * kXTileB + 2 * kWTileB];  // [X0][X1][W0][W1]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave & 1, wm = wave >> 1;
  const int n0 = blockIdx.x * kBNc;
  const int64_t m0 = (int64_t)blockIdx.y * kBM;
  const int col = lane & 31, kb = lane >> 5;

  // ---- tile loaders (global -> LDS without registers); the swizzle is applied on the global side ----
  const int64_t rows_left = M - m0;  // rows of x that exist from m0 on (>= 1)
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(x + (size_t)m0 * K), 0, (int)min((int64_t)kBM, rows_left) * K * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t w_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)(w + n0), 0, (int)(((size_t)K * N - n0) * 2), 0x00020000);
  // X tile: wave fills rows [32 wave, +32), 8 rows (1 KiB) per instruction; lane -> (row, physical chunk lane % 8)
  int xoff[4], woff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 32 * wave + 8 * i + (lane >> 3);
    xoff[i] = r * K * 2 + (((lane & 7) ^ swz_x(r)) << 4);
  }
  // W tile: wave fills rows [16 wave, +16), 4 rows per instruction; lane -> (row, physical chunk lane % 16)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 16 * wave + 4 * i + (lane >> 4);
    woff[i] = r * N * 2 + (((lane & 15) ^ swz_w(r)) << 4);
  }
  const uint32_t lds0 = (uint32_t)(size_t)((AG_LDS uint8_t *)smem);
  auto issue = [&](int t) {  // k-tile t -> buffers t & 1
    const int xs = t * kBK * 2;        // byte offset of the k-tile inside a row of x
    const int ws = t * kBK * N * 2;    // byte offset of the k-tile's first row of w
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t dx = lds0 + (t & 1) * kXTileB + (32 * wave + 8 * i) * kXRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dx), "v"(xoff[i]), "s"(x_rsrc), "s"(xs) : "memory");
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t dw = lds0 + 2 * kXTileB + (t & 1) * kWTileB + (16 * wave + 4 * i) * kWRowB;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(dw), "v"(woff[i]), "s"(w_rsrc), "s"(ws) : "memory");
    }
  };

  // ---- loop-invariant LDS offsets of this lane's fragments ----
  // B operand (X^T): lane (token col, k half kb), slab sl: 16 bytes at row 64 wm + 32 mt + col, chunk 2 sl + kb
  int x_off[2][4];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
      const int r = 64 * wm + 32 * mt + col;
      x_off[mt][sl] = r * kXRowB + (((2 * sl + kb) ^ swz_x(r)) << 4);
    }
  // A operand (W^T) by transposing reads: 16-lane group gl covers columns 16 (gl % 2) + 0..15 of a 32-column
  // sub-tile and k half gl / 2; lane i supplies the address of row 8 (gl / 2) + i / 4 (+ 4), columns 4 (i % 4) .. +3
  const int gl = lane >> 4, li = lane & 15;
  int w_off[2][2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const int r = 8 * (gl >> 1) + (li >> 2) + 4 * h2;                       // row inside a 16-k slab
      const int c = 4 * (2 * wn + nt) + 2 * (gl & 1) + ((li & 3) >> 1);       // 16-byte chunk of the 256-byte row
      w_off[nt][h2] = r * kWRowB + ((c ^ swz_w(r)) << 4) + (li & 1) * 8;
    }

  f32x16 acc[2][2];  // [nt][mt]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const int T = K / kBK;
  issue(0);
  for (int t = 0; t < T; ++t) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of tile t has landed
    __syncthreads();                                  // ... and everyone's; tile t - 1 is fully consumed
    if (t + 1 < T) issue(t + 1);
    const AG_LDS uint8_t *Xt = (const AG_LDS uint8_t *)smem + (t & 1) * kXTileB;
    const AG_LDS uint8_t *Wt = (const AG_LDS uint8_t *)smem + 2 * kXTileB + (t & 1) * kWTileB;
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        // swz_w only depends on the row inside the slab (r & 15), so the slab base can be added afterwards
        const AG_LDS uint8_t *base = Wt + 16 * sl * kWRowB;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(base + w_off[nt][0]));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((AG_LDS bf16x4 *)(base + w_off[nt][1]));
        a[nt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) b[mt] = *reinterpret_cast<const AG_LDS bf16x8 *>(Xt + x_off[mt][sl]);
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[nt], b[mt], acc[nt][mt], 0, 0, 0);
    }
  }

  // ---- epilogue: acc[nt][mt][r] = C[token m0 + 64 wm + 32 mt + col][n0 + 64 wn + 32 nt + 8 (r/4) + 4 kb + r%4] ----
  // The tile is one head of one projection: 128 tokens x 128 features = 128 whole output rows of 256 bytes.  A lane
  // owns 4-feature pieces of two tokens, so it would store scattered 8-byte pieces; the tile is laid out in the
  // (now unused) operand buffers instead, 16-byte chunks XOR-swizzled with the row, and leaves as whole rows, 4 per
  // instruction (lane -> row 4 i + lane / 16, chunk lane % 16), to the output and, for a kept token, to its cache row.
  const int hd = hp * kDh;
  const int which_t = n0 / hd, head_t = (n0 - which_t * hd) / kDh;
  __syncthreads();  // every wave is done with the last k-tile
  AG_LDS uint8_t *ost = (AG_LDS uint8_t *)smem;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int row = 64 * wm + 32 * mt + col;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x16 &c = acc[nt][mt];
        const u32x2 val = {pack2(c[4 * r4 + 0], c[4 * r4 + 1]), pack2(c[4 * r4 + 2], c[4 * r4 + 3])};
        *reinterpret_cast<AG_LDS u32x2 *>(ost + row * 256 + (((8 * wn + 4 * nt + r4) ^ (row & 15)) << 4) + 8 * kb) = val;
      }
  }
  __syncthreads();  // a row's two halves come from two waves
  const int ochunk = lane & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = 32 * wave + 4 * i + (lane >> 4);
    const int64_t m = m0 + row;
    const u32x4 val = *reinterpret_cast<const AG_LDS u32x4 *>(ost + row * 256 + ((ochunk ^ (row & 15)) << 4));
    if (m >= M) continue;
    const int64_t b = m / L, tt = m - b * L;
    uint16_t *dst = out + (((size_t)which_t * (M / L) * hp + (size_t)b * hp + head_t) * L + tt) * kDh + 8 * ochunk;
    *reinterpret_cast<u32x4 *>(dst) = val;
    if (COMPACT) {  // this token's row in the cache, if it is kept and fits
      const int u = (int)b * hp + head_t;
      const uint64_t word = cp.words[(size_t)u * cp.nw + (tt >> 6)];
      if ((word >> (tt & 63)) & 1ull) {
        const int c = cp.blk_off[(size_t)u * (cp.nw + 1) + (tt >> 6)] + __popcll(word & ((1ull << (tt & 63)) - 1ull));
        const int64_t r0 = cp.row_off[u], cap = cp.row_off[u + 1] - r0;
        if (c < cap) {
          uint16_t *crow = (which_t == 0 ? cp.kc : cp.vc) + (size_t)(r0 + c) * kDh;
          *reinterpret_cast<u32x4 *>(crow + 8 * ochunk) = val;
          if (which_t == 0 && ochunk == 0) cp.idx[r0 + c] = cp.pos0 + (int)tt;
        } else if (which_t == 0 && ochunk == 0) {
          atomicOr(cp.d_err, 1);  // the row is dropped, nothing is written out of bounds
        }
      }
    }
  }
  if (COMPACT && which_t == 0) {  // the K tile that holds a sequence's first token writes the unit's length
    const int64_t bb = (m0 + L - 1) / L + tid;  // thread t: the t-th sequence that starts inside this tile
    if (bb * L < m0 + kBM && bb * L < M) {
      const int u = (int)bb * hp + head_t;
      const int64_t cap = cp.row_off[u + 1] - cp.row_off[u];
      const int kept = cp.blk_off[(size_t)u * (cp.nw + 1) + cp.nw];
      cp.len[u] = (int)(kept < cap ? kept : cap);
    }
  }
}

}  // namespace

size_t ag_ws_gate_mha_bytes(int B, int L, int d_model, int hp, int H_f) {
  (void)d_model;
  const size_t tokens = (size_t)B * L;
  const int units = B * hp;
  ws_cursor count{nullptr, ~size_t(0) >> 1, 0, true};
  ag_pf_plan plan;
  float *part;
  ag_prefill_bf16_plan(1024, B, L, hp, hp, 128, count, &plan, &part);
  return 3 * ag_align256(tokens * hp * kDh * 2)      // Q', K', V'
         + ag_align256(tokens * hp * kDh * 2)        // attention output = gate features
         + ag_ws_scan_bytes(units, L) + ag_align256((size_t)(units + 1) * 8) + count.off +
         ag_ws_gate_bytes((int64_t)tokens, hp * kDh, H_f, AG_BF16) + 4096;
}

hipError_t ag_launch_gate_mha(ag_ctx *ctx, hipStream_t s, const void *x, int B, int L, int d_model, const void *w_qkv,
                              int hp, const void *w_o, const float *bias, int H_f, float thr, int n_sink, float scale,
                              float *logits, uint8_t *flags, ws_cursor &ws) {
  const int64_t tokens = (int64_t)B * L;
  const int units = B * hp, nw = ag_nwords(L), N = 3 * hp * kDh;
  const size_t per = (size_t)tokens * hp * kDh;
  uint16_t *qkv = ws.take<uint16_t>(3 * per);
  uint16_t *feat = ws.take<uint16_t>(per);
  uint64_t *words = ws.take<uint64_t>((size_t)units * nw);
  int32_t *blk_off = ws.take<int32_t>((size_t)units * (nw + 1));
  int64_t *row_off = ws.take<int64_t>(units + 1);
  ag_pf_plan plan;
  float *part = nullptr;
  ag_prefill_bf16_plan(ctx->num_cu, B, L, hp, hp, 128, ws, &plan, &part);
  if (!ws.ok) return hipSuccess;  // caller reports AG_EWORKSPACE

  AG_LAUNCH(ag_time_kernel(ctx, AG_K_MHA_PROJ), ag_proj_gemm_kernel<false>,
            dim3(N / kBNc, (unsigned)((tokens + kBM - 1) / kBM)), dim3(256), 0, s, (const uint16_t *)x,
            (const uint16_t *)w_qkv, tokens, d_model, N, L, hp, qkv, ag_proj_compact{});
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // every token is kept (no flags to read): mask words, prefix counts and the launch plan of the attention kernel
  if ((e = ag_launch_flag_scan(ctx, s, nullptr, units, L, words, blk_off, &plan)) != hipSuccess) return e;
  if ((e = ag_launch_slab_offsets(s, row_off, units, L)) != hipSuccess) return e;
  // every flag is set, so the compacted rows of a head are its K', V' rows themselves
  e = ag_launch_prefill_bf16(s, qkv, qkv + per, qkv + 2 * per, words, blk_off, B, L, hp, hp, 128, scale * 1.4426950408889634f,
                             1, qkv + per, qkv + 2 * per, row_off, feat, plan, part, /*out_token_major=*/true,
                             ag_time_kernel(ctx, AG_K_MHA_ATTN));
  if (e != hipSuccess) return e;
  return ag_launch_gate(ctx, s, feat, AG_BF16, B, L, hp * kDh, w_o, bias, H_f, thr, n_sink, logits, flags, ws);
}

// K/V projection with the compaction in its epilogue.  k_out and v_out must be one allocation of two
// [B, Hkv, L, 128] tensors back to back (k first).
size_t ag_ws_project_compact_bytes(int units, int L) {
  return ag_ws_scan_bytes(units, L) + 4096;
}

hipError_t ag_launch_project_compact(ag_ctx *ctx, hipStream_t s, const void *x, int B, int L, int d_model,
                                     const void *w_kv, int Hkv, const uint8_t *flags, int pos0, void *kv_out,
                                     void *kc, void *vc, int32_t *idx, const int64_t *row_off, int32_t *len,
                                     ws_cursor &ws) {
  const int64_t tokens = (int64_t)B * L;
  const int units = B * Hkv, nw = ag_nwords(L), N = 2 * Hkv * kDh;
  uint64_t *words = ws.take<uint64_t>((size_t)units * nw);
  int32_t *blk_off = ws.take<int32_t>((size_t)units * (nw + 1));
  if (!ws.ok) return hipSuccess;  // caller reports AG_EWORKSPACE
  hipError_t e = ag_launch_flag_scan(ctx, s, flags, units, L, words, blk_off, nullptr);
  if (e != hipSuccess) return e;
  const ag_proj_compact cp{words, blk_off, row_off, (uint16_t *)kc, (uint16_t *)vc, idx, len, ctx->d_err, nw, pos0};
  AG_LAUNCH(ag_time_kernel(ctx, AG_K_MHA_PROJ), ag_proj_gemm_kernel<true>,
            dim3(N / kBNc, (unsigned)((tokens + kBM - 1) / kBM)), dim3(256), 0, s, (const uint16_t *)x,
            (const uint16_t *)w_kv, tokens, d_model, N, L, Hkv, (uint16_t *)kv_out, cp);
  return hipGetLastError();
}
