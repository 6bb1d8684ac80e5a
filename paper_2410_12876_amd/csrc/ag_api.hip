// C ABI of libag: contexts, argument validation, workspace carving, kernel sequencing.
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <new>

#include "ag_internal.h"

bool ag_decode_supported(ag_dtype dt, int D, int G, int units);
bool ag_prefill_supported(ag_dtype dt, int D, int G);

ag_status ag_fail(ag_ctx *ctx, ag_status st, const char *fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

namespace {

constexpr int kMaxL = 1 << 22;

#define AG_REQUIRE(cond, st, ...) \
  do {                            \
    if (!(cond)) return ag_fail(ctx, st, __VA_ARGS__); \
  } while (0)

#define AG_HIP(call)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) return ag_fail(ctx, AG_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

bool dtype_ok(int dt) { return dt == AG_F32 || dt == AG_BF16; }

ag_status check_cache(ag_ctx *ctx, const ag_kv_cache *c) {
  AG_REQUIRE(c->k && c->v && c->idx && c->row_off && c->len, AG_EINVAL, "cache: null pointer");
  AG_REQUIRE(c->B > 0 && c->Hkv > 0 && c->D > 0, AG_EINVAL, "cache: B, Hkv, D must be positive");
  AG_REQUIRE(c->total_rows >= 0, AG_EINVAL, "cache: total_rows is negative");
  AG_REQUIRE(dtype_ok(c->dtype), AG_EINVAL, "cache: unknown dtype %d", (int)c->dtype);
  AG_REQUIRE((c->D * ag_dtype_size(c->dtype)) % 16 == 0, AG_EUNSUPPORTED, "cache: row size must be a multiple of 16 bytes");
  return AG_OK;
}

ws_cursor cursor(ag_ctx *ctx) { return ws_cursor{ctx->ws, ctx->ws_bytes, 0, true}; }

ag_status need_device(ag_ctx *ctx) {
  if (ctx->device < 0) return ag_fail(ctx, AG_EHIP, "context has no device (created with device = -1)");
  hipError_t e = hipSetDevice(ctx->device);
  if (e != hipSuccess) return ag_fail(ctx, AG_EHIP, "hipSetDevice(%d): %s", ctx->device, hipGetErrorString(e));
  return AG_OK;
}

}  // namespace

constexpr size_t kTailBytes = 256 + kGateTickets * sizeof(int32_t);

extern "C" {

ag_status ag_create(ag_ctx **out, int device, size_t workspace_bytes) {
  if (!out) return AG_EINVAL;
  *out = nullptr;
  ag_ctx *ctx = new (std::nothrow) ag_ctx();
  if (!ctx) return AG_EHIP;
  memset(ctx, 0, sizeof(*ctx));
  ctx->device = device;
  ctx->num_cu = 256;
  if (device >= 0) {
    hipDeviceProp_t prop;
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e == hipSuccess) {
      ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
      ctx->ws_bytes = ag_align256(workspace_bytes);
      e = hipMalloc((void **)&ctx->ws, ctx->ws_bytes + kTailBytes);
    }
    if (e == hipSuccess) {  // behind the workspace: the error word and the gate's arrival counters, all zero
      ctx->d_err = reinterpret_cast<int32_t *>(ctx->ws + ctx->ws_bytes);
      ctx->gate_tickets = reinterpret_cast<int32_t *>(ctx->ws + ctx->ws_bytes + 256);
      e = hipMemset(ctx->d_err, 0, kTailBytes);
    }
    if (e == hipSuccess) e = ag_static_scratch(device, &ctx->static_scratch);
    if (e != hipSuccess) {
      if (ctx->ws) (void)hipFree(ctx->ws);
      delete ctx;
      return AG_EHIP;
    }
  } else if (device == -1) {
    ctx->ws_bytes = ag_align256(workspace_bytes);  // sizes are still checked; nothing is allocated
  } else {
    delete ctx;
    return AG_EINVAL;
  }
  *out = ctx;
  return AG_OK;
}

void ag_destroy(ag_ctx *ctx) {
  if (!ctx) return;
  if (ctx->device >= 0 && ctx->ws) {
    (void)hipSetDevice(ctx->device);
    for (int id = 0; id < AG_K_COUNT; ++id) {
      ag_timer &t = ctx->timers[id];
      if (!t.start) continue;
      for (int i = 0; i < kTimerSlots; ++i) {
        (void)hipEventDestroy(t.start[i]);
        (void)hipEventDestroy(t.stop[i]);
      }
      delete[] t.start;
      delete[] t.stop;
    }
    (void)hipFree(ctx->ws);
  }
  delete ctx;
}

static const char *const kKernelNames[AG_K_COUNT] = {"gate", "gate_finalize", "flag_scan", "compact",
                                                     "prefill", "decode_partial", "decode_merge",
                                                     "mha_proj", "mha_attn", "norm_gate"};

int ag_timing_kernels(void) { return AG_K_COUNT; }

const char *ag_timing_kernel_name(int kernel_id) {
  return kernel_id >= 0 && kernel_id < AG_K_COUNT ? kKernelNames[kernel_id] : "";
}

ag_status ag_timing_enable(ag_ctx *ctx, int on) {
  if (!ctx) return AG_EINVAL;
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  if (on) {
    for (int id = 0; id < AG_K_COUNT; ++id) {
      ag_timer &t = ctx->timers[id];
      if (!t.start) {
        t.start = new (std::nothrow) hipEvent_t[kTimerSlots];
        t.stop = new (std::nothrow) hipEvent_t[kTimerSlots];
        if (!t.start || !t.stop) return ag_fail(ctx, AG_EHIP, "ag_timing_enable: out of host memory");
        for (int i = 0; i < kTimerSlots; ++i) {
          AG_HIP(hipEventCreate(&t.start[i]));
          AG_HIP(hipEventCreate(&t.stop[i]));
        }
      }
      t.n = 0;
    }
  }
  ctx->timing = on != 0;
  return AG_OK;
}

ag_status ag_timing_read(ag_ctx *ctx, int kernel_id, double *total_ms, int *launches) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(kernel_id >= 0 && kernel_id < AG_K_COUNT && total_ms && launches, AG_EINVAL,
             "ag_timing_read: bad kernel id or null pointer");
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  const ag_timer &t = ctx->timers[kernel_id];
  double sum = 0.0;
  for (int i = 0; i < t.n; ++i) {
    float ms = 0.f;
    AG_HIP(hipEventSynchronize(t.stop[i]));
    AG_HIP(hipEventElapsedTime(&ms, t.start[i], t.stop[i]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = t.n;
  return AG_OK;
}

const char *ag_last_error(const ag_ctx *ctx) { return ctx ? ctx->err : "null context"; }

size_t ag_workspace_bytes(int B, int L, int Hq, int Hkv, int D, ag_dtype dtype, int d_in, int64_t cache_rows) {
  if (B <= 0 || L <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv) return 0;
  const int units = B * Hkv;
  const size_t scan = ag_ws_scan_bytes(units, L);
  const size_t gate = d_in > 0 ? ag_ws_gate_bytes((int64_t)B * L, d_in, Hkv, dtype) : 0;
  // prefill without a cache compacts into the workspace: K, V rows, idx, row_off, len
  const size_t rows = (size_t)units * L;
  size_t plan_bytes = 0;
  if (dtype == AG_BF16 && (D == 128 || D == 64)) {  // sizes only: a cursor over no memory counts what the plan would take
    ws_cursor count{nullptr, ~size_t(0) >> 1, 0, true};
    ag_pf_plan plan;
    float *part;
    ag_prefill_bf16_plan(1024 /* upper bound on CUs: the split only shrinks with fewer */, B, L, Hq, Hkv, D, count,
                         &plan, &part);
    plan_bytes = count.off;
  }
  const size_t prefill = scan + 2 * ag_align256(rows * D * ag_dtype_size(dtype)) + ag_align256(rows * 4) +
                         ag_align256((size_t)(units + 1) * 8) + ag_align256((size_t)units * 4) +
                         plan_bytes;
  const size_t decode = cache_rows > 0 ? ag_ws_decode_bytes(units, Hq / Hkv, D, cache_rows) : 0;
  size_t need = scan;
  if (gate > need) need = gate;
  if (prefill > need) need = prefill;
  if (decode > need) need = decode;
  return need + 4096;
}

ag_status ag_poll_error(ag_ctx *ctx, void *hip_stream) {
  if (!ctx) return AG_EINVAL;
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  int32_t h = 0;
  AG_HIP(hipMemcpyAsync(&h, ctx->d_err, sizeof(h), hipMemcpyDeviceToHost, (hipStream_t)hip_stream));
  AG_HIP(hipStreamSynchronize((hipStream_t)hip_stream));
  if (h) {
    AG_HIP(hipMemsetAsync(ctx->d_err, 0, sizeof(h), (hipStream_t)hip_stream));
    AG_HIP(hipStreamSynchronize((hipStream_t)hip_stream));
    return ag_fail(ctx, AG_ECAPACITY, "a cache unit overflowed its capacity; the extra rows were dropped");
  }
  return AG_OK;
}

ag_status ag_gate(ag_ctx *ctx, void *hip_stream, const void *feat, ag_dtype dtype, int B, int L, int d_in,
                  const void *w_gate, const float *bias, int H_f, float tau, int n_sink, float *logits_out,
                  uint8_t *flags_out) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(feat && w_gate && bias && flags_out, AG_EINVAL, "ag_gate: null pointer");
  AG_REQUIRE(B > 0 && L > 0 && d_in > 0 && H_f > 0, AG_EINVAL, "ag_gate: B, L, d_in, H_f must be positive");
  AG_REQUIRE(tau > 0.f && tau < 1.f, AG_EINVAL, "ag_gate: tau must lie in (0, 1)");
  AG_REQUIRE(n_sink >= 0, AG_EINVAL, "ag_gate: n_sink is negative");
  AG_REQUIRE(dtype_ok(dtype), AG_EINVAL, "ag_gate: unknown dtype %d", (int)dtype);
  AG_REQUIRE(H_f <= 32, AG_EUNSUPPORTED, "ag_gate: H_f = %d exceeds 32", H_f);
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_gate: L = %d exceeds %d", L, kMaxL);
  AG_REQUIRE(dtype != AG_BF16 || d_in % 64 == 0, AG_EUNSUPPORTED, "ag_gate: bf16 needs d_in %% 64 == 0 (got %d)", d_in);
  AG_REQUIRE(ag_ws_gate_bytes((int64_t)B * L, d_in, H_f, dtype) <= ctx->ws_bytes, AG_EWORKSPACE,
             "ag_gate: workspace of %zu bytes is too small", ctx->ws_bytes);
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  const float thr = (float)log((double)tau / (1.0 - (double)tau));
  ws_cursor ws = cursor(ctx);
  hipError_t e = ag_launch_gate(ctx, (hipStream_t)hip_stream, feat, dtype, B, L, d_in, w_gate, bias, H_f, thr,
                                n_sink, logits_out, flags_out, ws);
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_gate: workspace of %zu bytes is too small (need %zu)", ctx->ws_bytes, ws.off);
  AG_HIP(e);
  return AG_OK;
}

ag_status ag_rmsnorm_gate(ag_ctx *ctx, void *hip_stream, const void *h, ag_dtype dtype, int B, int L, int d_in,
                          const void *norm_w, float eps, const void *w_gate, const float *bias, int H_f, float tau,
                          int n_sink, void *x_out, float *logits_out, uint8_t *flags_out) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(h && norm_w && w_gate && bias && x_out && flags_out, AG_EINVAL, "ag_rmsnorm_gate: null pointer");
  AG_REQUIRE(B > 0 && L > 0 && d_in > 0 && H_f > 0, AG_EINVAL, "ag_rmsnorm_gate: B, L, d_in, H_f must be positive");
  AG_REQUIRE(tau > 0.f && tau < 1.f, AG_EINVAL, "ag_rmsnorm_gate: tau must lie in (0, 1)");
  AG_REQUIRE(eps > 0.f, AG_EINVAL, "ag_rmsnorm_gate: eps must be positive");
  AG_REQUIRE(n_sink >= 0, AG_EINVAL, "ag_rmsnorm_gate: n_sink is negative");
  AG_REQUIRE(dtype_ok(dtype), AG_EINVAL, "ag_rmsnorm_gate: unknown dtype %d", (int)dtype);
  AG_REQUIRE(dtype == AG_BF16, AG_EUNSUPPORTED, "ag_rmsnorm_gate: only bf16 is built");
  AG_REQUIRE(d_in % 64 == 0 && d_in <= 8192, AG_EUNSUPPORTED,
             "ag_rmsnorm_gate: d_in must be a multiple of 64 and at most 8192 (got %d)", d_in);
  AG_REQUIRE(H_f <= 32, AG_EUNSUPPORTED, "ag_rmsnorm_gate: H_f = %d exceeds 32", H_f);
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_rmsnorm_gate: L = %d exceeds %d", L, kMaxL);
  AG_REQUIRE(((uintptr_t)h & 15) == 0 && ((uintptr_t)x_out & 15) == 0 && ((uintptr_t)norm_w & 15) == 0, AG_EINVAL,
             "ag_rmsnorm_gate: h, x_out and norm_w must be 16-byte aligned");
  AG_REQUIRE(ag_ws_gate_bytes((int64_t)B * L, d_in, H_f, dtype) <= ctx->ws_bytes, AG_EWORKSPACE,
             "ag_rmsnorm_gate: workspace of %zu bytes is too small", ctx->ws_bytes);
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  const float thr = (float)log((double)tau / (1.0 - (double)tau));
  ws_cursor ws = cursor(ctx);
  hipError_t e = ag_launch_norm_gate(ctx, (hipStream_t)hip_stream, h, B, L, d_in, norm_w, eps, w_gate, bias, H_f, thr,
                                     n_sink, x_out, logits_out, flags_out, ws);
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_rmsnorm_gate: workspace of %zu bytes is too small (need %zu)", ctx->ws_bytes,
             ws.off);
  AG_HIP(e);
  return AG_OK;
}

size_t ag_gate_mha_workspace_bytes(int B, int L, int d_model, int h_prime, int d_prime, int H_f) {
  if (B <= 0 || L <= 0 || d_model <= 0 || h_prime <= 0 || d_prime != 128 || H_f <= 0) return 0;
  return ag_ws_gate_mha_bytes(B, L, d_model, h_prime, H_f);
}

ag_status ag_gate_mha(ag_ctx *ctx, void *hip_stream, const void *x, ag_dtype dtype, int B, int L, int d_model,
                      const void *w_qkv, int h_prime, int d_prime, const void *w_o, const float *bias, int H_f,
                      float tau, int n_sink, float *logits_out, uint8_t *flags_out) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(x && w_qkv && w_o && bias && flags_out, AG_EINVAL, "ag_gate_mha: null pointer");
  AG_REQUIRE(B > 0 && L > 0 && d_model > 0 && h_prime > 0 && d_prime > 0 && H_f > 0, AG_EINVAL,
             "ag_gate_mha: sizes must be positive");
  AG_REQUIRE(tau > 0.f && tau < 1.f, AG_EINVAL, "ag_gate_mha: tau must lie in (0, 1)");
  AG_REQUIRE(n_sink >= 0, AG_EINVAL, "ag_gate_mha: n_sink is negative");
  AG_REQUIRE(dtype_ok(dtype), AG_EINVAL, "ag_gate_mha: unknown dtype %d", (int)dtype);
  AG_REQUIRE(dtype == AG_BF16 && d_prime == 128, AG_EUNSUPPORTED, "ag_gate_mha: only bf16 with d_prime = 128 is built");
  AG_REQUIRE(d_model % 64 == 0, AG_EUNSUPPORTED, "ag_gate_mha: d_model %% 64 != 0 (got %d)", d_model);
  AG_REQUIRE(H_f <= 32, AG_EUNSUPPORTED, "ag_gate_mha: H_f = %d exceeds 32", H_f);
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_gate_mha: L = %d exceeds %d", L, kMaxL);
  AG_REQUIRE((int64_t)B * h_prime <= 65535 && (int64_t)d_model * 3 * h_prime * 128 < (1ll << 30) &&
                 (int64_t)B * L < (1ll << 31) - 128,
             AG_EUNSUPPORTED, "ag_gate_mha: problem too large");
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  const float thr = (float)log((double)tau / (1.0 - (double)tau));
  ws_cursor ws = cursor(ctx);
  hipError_t e = ag_launch_gate_mha(ctx, (hipStream_t)hip_stream, x, B, L, d_model, w_qkv, h_prime, w_o, bias, H_f, thr,
                                    n_sink, 1.0f / sqrtf((float)d_prime), logits_out, flags_out, ws);
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_gate_mha: workspace of %zu bytes is too small (need %zu)", ctx->ws_bytes, ws.off);
  AG_HIP(e);
  return AG_OK;
}

ag_status ag_compact_kv(ag_ctx *ctx, void *hip_stream, const void *k, const void *v, const uint8_t *flags, int L,
                        int pos0, ag_kv_cache *cache) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(k && v && flags && cache, AG_EINVAL, "ag_compact_kv: null pointer");
  AG_REQUIRE(L > 0, AG_EINVAL, "ag_compact_kv: L must be positive");
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_compact_kv: L = %d exceeds %d", L, kMaxL);
  ag_status st = check_cache(ctx, cache);
  if (st != AG_OK) return st;
  const int units = cache->B * cache->Hkv;
  AG_REQUIRE(ag_ws_scan_bytes(units, L) <= ctx->ws_bytes, AG_EWORKSPACE,
             "ag_compact_kv: workspace of %zu bytes is too small", ctx->ws_bytes);
  st = need_device(ctx);
  if (st != AG_OK) return st;
  const int nw = ag_nwords(L);
  ws_cursor ws = cursor(ctx);
  uint64_t *words = ws.take<uint64_t>((size_t)units * nw);
  int32_t *blk_off = ws.take<int32_t>((size_t)units * (nw + 1));
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_compact_kv: workspace too small (need %zu)", ws.off);
  hipStream_t s = (hipStream_t)hip_stream;
  AG_HIP(ag_launch_scan_compact(ctx, s, flags, units, L, words, blk_off, nullptr, k, v,
                                (int)(cache->D * ag_dtype_size(cache->dtype)), pos0, cache->k, cache->v, cache->idx,
                                cache->row_off, cache->len));
  return AG_OK;
}

ag_status ag_pack_row_off(ag_ctx *ctx, void *hip_stream, const uint8_t *flags, int B, int Hkv, int L, int room,
                          int64_t total_rows, int64_t *row_off, int64_t *rows_needed) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(flags && row_off, AG_EINVAL, "ag_pack_row_off: null pointer");
  AG_REQUIRE(B > 0 && Hkv > 0 && L > 0, AG_EINVAL, "ag_pack_row_off: B, Hkv, L must be positive");
  AG_REQUIRE(room >= 0 && total_rows >= 0, AG_EINVAL, "ag_pack_row_off: room and total_rows must not be negative");
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_pack_row_off: L = %d exceeds %d", L, kMaxL);
  AG_REQUIRE((int64_t)B * Hkv <= 65535, AG_EUNSUPPORTED, "ag_pack_row_off: B * Hkv exceeds 65535");
  const int units = B * Hkv;
  ws_cursor ws = cursor(ctx);
  int32_t *kept = ws.take<int32_t>(units);
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_pack_row_off: workspace of %zu bytes is too small (need %zu)", ctx->ws_bytes, ws.off);
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  AG_HIP(ag_launch_pack_row_off((hipStream_t)hip_stream, flags, units, L, room, total_rows, kept, row_off, rows_needed));
  return AG_OK;
}

size_t ag_project_compact_workspace_bytes(int B, int L, int Hkv) {
  if (B <= 0 || L <= 0 || Hkv <= 0) return 0;
  return ag_ws_project_compact_bytes(B * Hkv, L);
}

ag_status ag_project_compact_kv(ag_ctx *ctx, void *hip_stream, const void *x, ag_dtype dtype, int B, int L,
                                int d_model, const void *w_kv, const uint8_t *flags, int pos0, void *kv_out,
                                ag_kv_cache *cache) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(x && w_kv && flags && kv_out && cache, AG_EINVAL, "ag_project_compact_kv: null pointer");
  AG_REQUIRE(B > 0 && L > 0 && d_model > 0, AG_EINVAL, "ag_project_compact_kv: B, L, d_model must be positive");
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_project_compact_kv: L = %d exceeds %d", L, kMaxL);
  ag_status st = check_cache(ctx, cache);
  if (st != AG_OK) return st;
  AG_REQUIRE(cache->B == B, AG_EINVAL, "ag_project_compact_kv: cache->B = %d but B = %d", cache->B, B);
  AG_REQUIRE(dtype == AG_BF16 && cache->dtype == AG_BF16 && cache->D == 128, AG_EUNSUPPORTED,
             "ag_project_compact_kv: bf16 with head size 128 only");
  AG_REQUIRE(d_model % 64 == 0, AG_EUNSUPPORTED, "ag_project_compact_kv: d_model %% 64 != 0 (got %d)", d_model);
  AG_REQUIRE((int64_t)B * L * d_model * 2 < (int64_t)1 << 31 && (int64_t)d_model * 2 * cache->Hkv * 128 * 2 < (int64_t)1 << 31,
             AG_EUNSUPPORTED, "ag_project_compact_kv: x or w_kv exceeds 2 GiB (the tile loaders use 32-bit offsets)");
  const int units = B * cache->Hkv;
  AG_REQUIRE(ag_ws_project_compact_bytes(units, L) <= ctx->ws_bytes, AG_EWORKSPACE,
             "ag_project_compact_kv: workspace of %zu bytes is too small", ctx->ws_bytes);
  st = need_device(ctx);
  if (st != AG_OK) return st;
  ws_cursor ws = cursor(ctx);
  hipError_t e = ag_launch_project_compact(ctx, (hipStream_t)hip_stream, x, B, L, d_model, w_kv, cache->Hkv, flags, pos0,
                                           kv_out, cache->k, cache->v, cache->idx, cache->row_off, cache->len, ws);
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_project_compact_kv: workspace too small (need %zu)", ws.off);
  AG_HIP(e);
  return AG_OK;
}

ag_status ag_prefill_attn(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                          const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype, float scale,
                          const ag_kv_cache *cache, void *out) {
  return ag_prefill_attn_recent(ctx, hip_stream, q, k, v, flags, B, L, Hq, Hkv, D, dtype, scale, cache, 1, out);
}

}  // extern "C"

namespace {
// ag_prefill_attn[_recent] (fill_cache == false: `cache`, if given, already holds the compacted rows) and
// ag_compact_prefill_attn (fill_cache == true: the call's own scan also drives the compaction into `cache`).
ag_status prefill_common(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                         const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype, float scale,
                         const ag_kv_cache *cache, int n_recent, void *out, bool fill_cache, int pos0) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(!fill_cache || cache, AG_EINVAL, "ag_compact_prefill_attn: cache is NULL");
  AG_REQUIRE(n_recent >= 1 && n_recent <= 64, AG_EINVAL, "ag_prefill_attn: n_recent = %d outside [1, 64]", n_recent);
  AG_REQUIRE(q && k && v && flags && out, AG_EINVAL, "ag_prefill_attn: null pointer");
  AG_REQUIRE(B > 0 && L > 0 && Hq > 0 && Hkv > 0 && D > 0, AG_EINVAL, "ag_prefill_attn: sizes must be positive");
  AG_REQUIRE(Hq % Hkv == 0, AG_EINVAL, "ag_prefill_attn: Hq %% Hkv != 0");
  AG_REQUIRE(scale > 0.f && isfinite(scale), AG_EINVAL, "ag_prefill_attn: scale must be positive and finite");
  AG_REQUIRE(dtype_ok(dtype), AG_EINVAL, "ag_prefill_attn: unknown dtype %d", (int)dtype);
  AG_REQUIRE(L <= kMaxL, AG_EUNSUPPORTED, "ag_prefill_attn: L = %d exceeds %d", L, kMaxL);
  AG_REQUIRE(ag_prefill_supported(dtype, D, Hq / Hkv), AG_EUNSUPPORTED,
             "ag_prefill_attn: unsupported dtype/D/group (%d, %d, %d)", (int)dtype, D, Hq / Hkv);
  AG_REQUIRE((int64_t)B * Hq <= 65535, AG_EUNSUPPORTED, "ag_prefill_attn: B * Hq exceeds 65535");
  if (cache) {
    ag_status st = check_cache(ctx, cache);
    if (st != AG_OK) return st;
    AG_REQUIRE(cache->B == B && cache->Hkv == Hkv && cache->D == D && cache->dtype == dtype, AG_EINVAL,
               "ag_prefill_attn: cache shape or dtype differs from the call's");
  }
  const int units = B * Hkv;
  const int nw = ag_nwords(L);
  const size_t esz = ag_dtype_size(dtype);
  ws_cursor ws = cursor(ctx);
  uint64_t *words = ws.take<uint64_t>((size_t)units * nw);
  int32_t *blk_off = ws.take<int32_t>((size_t)units * (nw + 1));
  const void *kc, *vc;
  const int64_t *row_off;
  char *wk = nullptr, *wv = nullptr;
  int32_t *widx = nullptr, *wlen = nullptr;
  int64_t *wro = nullptr;
  if (cache) {
    kc = cache->k; vc = cache->v; row_off = cache->row_off;
  } else {
    wk = ws.take<char>((size_t)units * L * D * esz);
    wv = ws.take<char>((size_t)units * L * D * esz);
    widx = ws.take<int32_t>((size_t)units * L);
    wro = ws.take<int64_t>(units + 1);
    wlen = ws.take<int32_t>(units);
    kc = wk; vc = wv; row_off = wro;
  }
  ag_pf_plan plan;
  memset(&plan, 0, sizeof(plan));
  float *part = nullptr;
  const bool tuned = dtype == AG_BF16;  // (D = 128 or 64: ag_prefill_supported)
  if (tuned) ag_prefill_bf16_plan(ctx->num_cu, B, L, Hq, Hkv, D, ws, &plan, &part);
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_prefill_attn: workspace of %zu bytes is too small (need %zu)", ctx->ws_bytes,
             ws.off);
  ag_status st = need_device(ctx);
  if (st != AG_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  const ag_pf_plan *pl = tuned ? &plan : nullptr;
  if (!cache) {  // scan and compaction in one launch, into the workspace
    AG_HIP(ag_launch_slab_offsets(s, wro, units, L));
    AG_HIP(ag_launch_scan_compact(ctx, s, flags, units, L, words, blk_off, pl, k, v, (int)(D * esz), 0, wk, wv, widx, wro,
                                  wlen));
  } else if (fill_cache) {  // ... into the caller's cache
    AG_HIP(ag_launch_scan_compact(ctx, s, flags, units, L, words, blk_off, pl, k, v, (int)(D * esz), pos0, cache->k,
                                  cache->v, cache->idx, cache->row_off, cache->len));
  } else {  // the cache already holds the compacted rows
    AG_HIP(ag_launch_flag_scan(ctx, s, flags, units, L, words, blk_off, pl));
  }
  AG_HIP(ag_launch_prefill(ctx, s, q, k, v, words, blk_off, B, L, Hq, Hkv, D, dtype, scale, n_recent, kc, vc, row_off,
                           out, plan, part));
  return AG_OK;
}
}  // namespace

extern "C" {

ag_status ag_prefill_attn_recent(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                                 const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype,
                                 float scale, const ag_kv_cache *cache, int n_recent, void *out) {
  return prefill_common(ctx, hip_stream, q, k, v, flags, B, L, Hq, Hkv, D, dtype, scale, cache, n_recent, out, false, 0);
}

ag_status ag_compact_prefill_attn(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                                  const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype,
                                  float scale, int pos0, ag_kv_cache *cache, int n_recent, void *out) {
  return prefill_common(ctx, hip_stream, q, k, v, flags, B, L, Hq, Hkv, D, dtype, scale, cache, n_recent, out, true,
                        pos0);
}

namespace {
ag_status check_ring(ag_ctx *ctx, const ag_recent_ring *r) {
  AG_REQUIRE(r->k && r->v && r->flags && r->pos, AG_EINVAL, "ring: null pointer");
  AG_REQUIRE(r->n_recent >= 2 && r->n_recent <= 64, AG_EINVAL, "ring: n_recent = %d outside [2, 64]", r->n_recent);
  return AG_OK;
}
ag_ring_dev ring_dev(const ag_recent_ring *r) {
  return r ? ag_ring_dev{r->k, r->v, r->flags, r->pos, r->n_recent} : ag_ring_dev{nullptr, nullptr, nullptr, nullptr, 0};
}
}  // namespace

ag_status ag_recent_fill(ag_ctx *ctx, void *hip_stream, const void *k, const void *v, const uint8_t *flags, int B,
                         int L, int Hkv, int D, ag_dtype dtype, int pos0, ag_recent_ring *ring) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(k && v && flags && ring, AG_EINVAL, "ag_recent_fill: null pointer");
  AG_REQUIRE(B > 0 && L > 0 && Hkv > 0 && D > 0 && pos0 >= 0, AG_EINVAL, "ag_recent_fill: bad sizes");
  AG_REQUIRE(dtype_ok(dtype), AG_EINVAL, "ag_recent_fill: unknown dtype %d", (int)dtype);
  ag_status st = check_ring(ctx, ring);
  if (st != AG_OK) return st;
  st = need_device(ctx);
  if (st != AG_OK) return st;
  AG_HIP(ag_launch_ring_fill((hipStream_t)hip_stream, k, v, flags, B * Hkv, L, D, dtype, pos0, ring_dev(ring)));
  return AG_OK;
}

ag_status ag_decode_attn(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                         const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache, void *out) {
  return ag_decode_attn_recent(ctx, hip_stream, q, k_new, v_new, new_flags, pos, Hq, scale, cache, nullptr, out);
}

}  // extern "C"

namespace {
// ag_decode_attn[_recent] (records in the context's workspace) and ag_decode_attn_static (records in the library's
// static per-GPU scratch array: nothing of the workspace is touched).
ag_status decode_common(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                        const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache,
                        ag_recent_ring *ring, void *out, bool static_scratch);
}  // namespace

extern "C" {

ag_status ag_decode_attn_recent(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                                const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache,
                                ag_recent_ring *ring, void *out) {
  return decode_common(ctx, hip_stream, q, k_new, v_new, new_flags, pos, Hq, scale, cache, ring, out, false);
}

size_t ag_decode_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t ag_decode_scratch_bytes(const ag_kv_cache *cache, int Hq) {
  if (!cache || cache->B <= 0 || cache->Hkv <= 0 || cache->D <= 0 || Hq <= 0 || Hq % cache->Hkv || cache->total_rows < 0)
    return 0;
  return ag_ws_decode_bytes(cache->B * cache->Hkv, Hq / cache->Hkv, cache->D, cache->total_rows);
}

ag_status ag_decode_attn_static(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                                const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache,
                                void *out) {
  return decode_common(ctx, hip_stream, q, k_new, v_new, new_flags, pos, Hq, scale, cache, nullptr, out, true);
}

}  // extern "C"

namespace {
ag_status decode_common(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                        const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache,
                        ag_recent_ring *ring, void *out, bool static_scratch) {
  if (!ctx) return AG_EINVAL;
  AG_REQUIRE(q && k_new && v_new && cache && out, AG_EINVAL, "ag_decode_attn: null pointer");
  ag_status st = check_cache(ctx, cache);
  if (st != AG_OK) return st;
  if (ring) {
    st = check_ring(ctx, ring);
    if (st != AG_OK) return st;
    AG_REQUIRE(pos >= 0, AG_EINVAL, "ag_decode_attn: pos must not be negative with a recent-token ring");
  }
  AG_REQUIRE(Hq > 0 && Hq % cache->Hkv == 0, AG_EINVAL, "ag_decode_attn: Hq must be a positive multiple of Hkv");
  AG_REQUIRE(scale > 0.f && isfinite(scale), AG_EINVAL, "ag_decode_attn: scale must be positive and finite");
  const int G = Hq / cache->Hkv, units = cache->B * cache->Hkv;
  AG_REQUIRE(ag_decode_supported(cache->dtype, cache->D, G, units), AG_EUNSUPPORTED,
             "ag_decode_attn: unsupported dtype/D/group/units (%d, %d, %d, %d)", (int)cache->dtype, cache->D, G, units);
  const size_t need = ag_ws_decode_bytes(units, G, cache->D, cache->total_rows);
  if (static_scratch)
    AG_REQUIRE(need <= kStaticScratchBytes, AG_EWORKSPACE,
               "ag_decode_attn_static: this cache needs %zu bytes of scratch, the static array holds %zu "
               "(ag_decode_scratch_bytes; use ag_decode_attn with a workspace instead)", need, kStaticScratchBytes);
  else
    AG_REQUIRE(need <= ctx->ws_bytes, AG_EWORKSPACE, "ag_decode_attn: workspace of %zu bytes is too small",
               ctx->ws_bytes);
  st = need_device(ctx);
  if (st != AG_OK) return st;
  ws_cursor ws = static_scratch ? ws_cursor{ctx->static_scratch, kStaticScratchBytes, 0, true} : cursor(ctx);
  hipError_t e = ag_launch_decode(ctx, (hipStream_t)hip_stream, q, k_new, v_new, new_flags, pos, cache->B, Hq, cache->Hkv,
                                  cache->D, cache->dtype, scale, cache->k, cache->v, cache->idx, cache->row_off,
                                  cache->len, cache->total_rows, out, ws, ring_dev(ring));
  AG_REQUIRE(ws.ok, AG_EWORKSPACE, "ag_decode_attn: workspace too small (need %zu)", ws.off);
  AG_HIP(e);
  return AG_OK;
}
}  // namespace
