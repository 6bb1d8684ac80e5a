// Internal declarations shared by the libag translation units (not part of the C ABI).
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "ag.h"
#include "ag_bench.h"

// Kernels that ag_timing_* can time (ids are part of the ABI, see ag_bench.h).
enum { AG_K_GATE = 0, AG_K_GATE_FINALIZE, AG_K_FLAG_SCAN, AG_K_COMPACT, AG_K_PREFILL, AG_K_DECODE_PARTIAL,
       AG_K_DECODE_MERGE, AG_K_MHA_PROJ, AG_K_MHA_ATTN, AG_K_NORM_GATE, AG_K_COUNT };
constexpr int kTimerSlots = 1024;  // launches remembered per kernel id
constexpr int kGateTickets = 1024; // token tiles whose K splits can be counted
constexpr size_t kStaticScratchBytes = size_t(16) << 20;  // per-GPU static scratch of ag_decode_attn_static

struct ag_timer {
  hipEvent_t *start, *stop;  // kTimerSlots each, created on first enable
  int n;                     // launches recorded since the last enable
};

struct ag_ctx {
  int device;       // -1: no device (argument validation only)
  int num_cu;
  char *ws;         // device workspace
  size_t ws_bytes;
  int32_t *d_err;   // sticky device error word (bit 0: cache capacity overflow)
  int32_t *gate_tickets;  // [kGateTickets] arrival counters of the gate's K splits: zero between launches
  char *static_scratch;   // this device's copy of the library's static scratch array (ag_decode_attn_static)
  bool timing;
  ag_timer timers[AG_K_COUNT];
  char err[320];
};

// Event pair around one kernel launch when timing is on (no-ops otherwise).
static inline void ag_tick(ag_ctx *ctx, int id, hipStream_t s) {
  if (ctx->timing && ctx->timers[id].n < kTimerSlots) (void)hipEventRecord(ctx->timers[id].start[ctx->timers[id].n], s);
}
static inline void ag_tock(ag_ctx *ctx, int id, hipStream_t s) {
  if (ctx->timing && ctx->timers[id].n < kTimerSlots) {
    (void)hipEventRecord(ctx->timers[id].stop[ctx->timers[id].n], s);
    ctx->timers[id].n++;
  }
}

// Events attached to ONE kernel launch (hipExtLaunchKernelGGL records them right at the kernel's start and end, so
// the duration is the kernel's own, without the few microseconds an event pair around a launch adds).  Both are
// null when timing is off or the slots are used up; AG_LAUNCH then launches the ordinary way.
struct ag_evpair {
  hipEvent_t start, stop;
};
static inline ag_evpair ag_time_kernel(ag_ctx *ctx, int id) {
  ag_evpair e{nullptr, nullptr};
  if (ctx && ctx->timing && ctx->timers[id].n < kTimerSlots) {
    e.start = ctx->timers[id].start[ctx->timers[id].n];
    e.stop = ctx->timers[id].stop[ctx->timers[id].n];
    ctx->timers[id].n++;
  }
  return e;
}
#define AG_LAUNCH(ev, kernel, grid, block, shmem, stream, ...)                                              \
  do {                                                                                                      \
    const ag_evpair ev_ = (ev); /* evaluated once: taking a pair uses up a timer slot */                    \
    if (ev_.start)                                                                                          \
      hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, ev_.start, ev_.stop, 0, __VA_ARGS__);       \
    else                                                                                                    \
      hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                  \
  } while (0)

// ---- How workgroups of ONE launch hand data to each other (prefill chunk states, gate K splits, the planner's
// per-unit counts) -------------------------------------------------------------------------------------------------
// Pattern: a producer writes its data, waits until those writes have completed, then bumps an arrival counter with an
// atomic add; the workgroup that sees the last arrival reads everybody's data.  What makes this hold on gfx950,
// instruction by instruction:
//   * The 8 XCDs have an L2 each, and those L2s are not kept coherent with one another inside a kernel; a plain store
//     may sit dirty in its XCD's L2 and a plain load may hit a stale line.  The data that is exchanged is therefore
//     written ONLY with system-scope atomic stores and read ONLY with system-scope atomic loads, which the compiler
//     turns into global_store / global_load with the sc0 and sc1 bits set (checked in the generated code): such a store
//     is written through to memory and such a load is served from memory, never from a line cached earlier.  That is
//     the per-access form of what a release fence (write back the whole L2) and an acquire fence (invalidate it) would
//     do for all lines -- and those two fences were measured to stall every workgroup of the XCD.
//   * s_waitcnt vmcnt(0) after the stores: a written-through store is counted as complete only when memory has
//     acknowledged it, so when the counter is bumped (by a thread of the same wave, or after a workgroup barrier that
//     follows every wave's own wait) the data is in memory.
//   * The counter itself is a device-scope atomic add (executed in memory-side atomic units, one copy for all XCDs).
//     The reader's loads are issued after its workgroup has seen the counter's value (a barrier in between), so they
//     come after the add in time, and being served from memory they observe everything written before it.
// In the language's terms the accesses are relaxed atomics ordered by that argument about the hardware, not by
// release/acquire semantics; the tests that alternate launches under concurrent memory traffic and compare bits guard it.

// Bump allocator over the context's workspace; every block is 256-byte aligned.
struct ws_cursor {
  char *base;
  size_t size, off;
  bool ok;
  template <typename T>
  T *take(size_t n) {
    size_t bytes = (n * sizeof(T) + 255) & ~size_t(255);
    if (off + bytes > size) { ok = false; off += bytes; return nullptr; }
    T *p = reinterpret_cast<T *>(base + off);
    off += bytes;
    return p;
  }
};

static inline size_t ag_align256(size_t b) { return (b + 255) & ~size_t(255); }
static inline size_t ag_dtype_size(ag_dtype t) { return t == AG_BF16 ? 2 : 4; }

ag_status ag_fail(ag_ctx *ctx, ag_status st, const char *fmt, ...);

// ---- sizes of the per-call workspace blocks (host helpers, also used by ag_workspace_bytes) ----
static inline int ag_nwords(int L) { return (L + 63) / 64; }
size_t ag_ws_scan_bytes(int units, int L);
size_t ag_ws_gate_bytes(int64_t tokens, int d_in, int H_f, ag_dtype dt);
size_t ag_ws_decode_bytes(int units, int G, int D, int64_t cache_rows);

// What the flag scan's last workgroup prepares for the bf16 prefill kernel (all pointers device, nullable):
// the head order that balances XCDs, the number of key tiles per chunk, and zeroed per-item arrival counters.
struct ag_pf_plan {
  int32_t *order;        // [n_hy] head block at each position of a query-tile row
  int32_t *chunk_tiles;  // [1]   key tiles per chunk, from the measured amount of work
  int32_t *tickets;      // [n_items] chunks of an item that have stored their partial state
  int32_t *kept;         // [units]  kept rows per unit, exchanged between the scan's workgroups
  int n_hy, HB, BM, n_items, n_split, slots, max_tiles;
  int NW;                // waves per workgroup of the prefill kernel (4 or 8)
  int head_major;        // block order of the prefill kernel: a head's query tiles together (many heads)
  int n_sp;              // query-tile rows (the longest ones) that can hold an item longer than one chunk
};

// ---- kernel launchers (each enqueues on `s` and returns the launch status) ----
// Flag scan: 64-bit keep masks per 64 tokens and their exclusive prefix counts.
//   words [units, nw], blk_off [units, nw + 1]  (nw = ceil(L / 64)); blk_off[u][nw] = kept rows of unit u.
hipError_t ag_launch_flag_scan(ag_ctx *ctx, hipStream_t s, const uint8_t *flags, int units, int L, uint64_t *words,
                               int32_t *blk_off, const ag_pf_plan *plan);

// row_off[u] = u * L for u in [0, units]: one full-length slab per unit.
hipError_t ag_launch_slab_offsets(hipStream_t s, int64_t *row_off, int units, int L);

// Packed cache layout: row_off[u + 1] = min(sum_{u' <= u} (kept flags of u' + room), total_rows); kept[units] is
// scratch; rows_needed (nullable) receives the unclamped total.
hipError_t ag_launch_pack_row_off(hipStream_t s, const uint8_t *flags, int units, int L, int room, int64_t total_rows,
                                  int32_t *kept, int64_t *row_off, int64_t *rows_needed);

// The scan above and the stable compaction of the kept K/V rows in one launch (timed as the compaction).
hipError_t ag_launch_scan_compact(ag_ctx *ctx, hipStream_t s, const uint8_t *flags, int units, int L, uint64_t *words,
                                  int32_t *blk_off, const ag_pf_plan *plan, const void *k, const void *v, int row_bytes,
                                  int pos0, void *kc, void *vc, int32_t *idx, const int64_t *row_off, int32_t *len);

hipError_t ag_launch_gate(ag_ctx *ctx, hipStream_t s, const void *feat, ag_dtype dt, int B, int L, int d_in,
                          const void *w, const float *bias, int H_f, float thr, int n_sink, float *logits,
                          uint8_t *flags, ws_cursor &ws);

hipError_t ag_launch_prefill(ag_ctx *ctx, hipStream_t s, const void *q, const void *k, const void *v,
                             const uint64_t *words, const int32_t *blk_off, int B, int L, int Hq, int Hkv, int D,
                             ag_dtype dt, float scale, int n_recent, const void *kc, const void *vc,
                             const int64_t *row_off, void *out, const ag_pf_plan &plan, float *part);

// bf16, D = 128 or 64: the kernel of ag_prefill_bf16.hip (qscale = scale * log2 e).  ag_prefill_bf16_plan carves
// the plan's buffers and the partial-state buffer out of the workspace (plan.n_split == 1: no key split).
void ag_prefill_bf16_plan(int num_cu, int B, int L, int Hq, int Hkv, int D, ws_cursor &ws, ag_pf_plan *plan,
                          float **part);
hipError_t ag_launch_prefill_bf16(hipStream_t s, const void *q, const void *k, const void *v, const uint64_t *words,
                                  const int32_t *blk_off, int B, int L, int Hq, int Hkv, int D, float qscale,
                                  int n_recent, const void *kc, const void *vc, const int64_t *row_off, void *out,
                                  const ag_pf_plan &plan, float *part, bool out_token_major = false,
                                  ag_evpair ev = ag_evpair{nullptr, nullptr});

// The 64-queries-per-wave variant of the same kernel (experiment, AG_PREFILL_Q64=1; n_recent = 1 only): same plan,
// same grid of `blocks` workgroups, 128 threads each.
hipError_t ag_launch_prefill_d128_q64(hipStream_t s, const void *q, const void *k, const void *v, const uint64_t *words,
                                      const int32_t *blk_off, int L, int Hq, int Hkv, float qscale, const void *kc,
                                      const void *vc, const int64_t *row_off, void *out, const ag_pf_plan &plan,
                                      float *part, bool out_token_major, ag_evpair ev, unsigned blocks);

// RMS normalisation of h (weights g, bf16, d_in <= 8192) fused with the gate; x_out may be h itself.
hipError_t ag_launch_norm_gate(ag_ctx *ctx, hipStream_t s, const void *h, int B, int L, int d_in, const void *g,
                               float eps, const void *w, const float *bias, int H_f, float thr, int n_sink,
                               void *x_out, float *logits, uint8_t *flags, ws_cursor &ws);

// The paper's main gate: MHA' (projection GEMM, causal attention with hp heads of 128) in front of ag_launch_gate.
size_t ag_ws_gate_mha_bytes(int B, int L, int d_model, int hp, int H_f);
hipError_t ag_launch_gate_mha(ag_ctx *ctx, hipStream_t s, const void *x, int B, int L, int d_model, const void *w_qkv,
                              int hp, const void *w_o, const float *bias, int H_f, float thr, int n_sink, float scale,
                              float *logits, uint8_t *flags, ws_cursor &ws);

// The layer's K/V projection (bf16, head size 128) with the compaction in the GEMM's epilogue.  kv_out = two
// [B, Hkv, L, 128] tensors back to back (k, then v).
size_t ag_ws_project_compact_bytes(int units, int L);
hipError_t ag_launch_project_compact(ag_ctx *ctx, hipStream_t s, const void *x, int B, int L, int d_model,
                                     const void *w_kv, int Hkv, const uint8_t *flags, int pos0, void *kv_out,
                                     void *kc, void *vc, int32_t *idx, const int64_t *row_off, int32_t *len,
                                     ws_cursor &ws);

// Device view of an ag_recent_ring (k == nullptr: no ring).  Slot w of unit u is element u * n + w.
struct ag_ring_dev {
  void *k, *v;      // [units, n, D]
  uint8_t *flags;   // [units, n]
  int32_t *pos;     // [units, n]
  int n;            // slots per unit = n_recent
};
constexpr int32_t kRingEmpty = -(1 << 30);  // position stored in an empty ring slot

hipError_t ag_launch_decode(ag_ctx *ctx, hipStream_t s, const void *q, const void *k_new, const void *v_new,
                            const uint8_t *new_flags, int pos, int B, int Hq, int Hkv, int D, ag_dtype dt,
                            float scale, void *kc, void *vc, int32_t *idx, const int64_t *row_off, int32_t *len,
                            int64_t total_rows, void *out, ws_cursor &ws, ag_ring_dev ring);

// Device address of the static scratch array (kStaticScratchBytes) on `device`; looked up once per device.
hipError_t ag_static_scratch(int device, char **ptr);

// Ring <- the last min(L, n) prompt tokens of every unit (k, v [units, L, D], flags [units, L]).
hipError_t ag_launch_ring_fill(hipStream_t s, const void *k, const void *v, const uint8_t *flags, int units, int L,
                               int D, ag_dtype dt, int pos0, ag_ring_dev ring);
