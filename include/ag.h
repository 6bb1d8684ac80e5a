/*
 * libag -- Attention-Gate (AG) KV-cache eviction, inference hot path, for AMD MI355X (gfx950).
 *
 * Four calls cover one attention layer:
 *   ag_gate          token features -> one logit per (token, head) -> keep/evict flags   (Eq. 3, Eq. 4)
 *   ag_compact_kv    keep only the flagged K/V rows, per (batch, KV head), in a ragged cache
 *                    (Sec. 3.3: k, v of a token are retained iff its flag is 1)
 *   ag_prefill_attn  causal attention under the flag mask with the diagonal kept       (Eq. 2, Eq. 5)
 *   ag_decode_attn   one decoding step over the ragged cache, then append             (Sec. 3.1)
 *
 * Conventions
 *   - Every tensor argument is caller-owned, contiguous DEVICE memory in the stated layout unless marked
 *     "host".  The library never frees or keeps caller memory.  Its only allocation is the workspace made by
 *     ag_create and released by ag_destroy.
 *   - Work is enqueued on the given HIP stream (a hipStream_t passed as void*; NULL = default stream) and the
 *     call returns without synchronising.  Calls on one stream are ordered.
 *   - The return value reports errors that can be seen from the host (bad arguments, unsupported shapes,
 *     workspace too small, launch failure).  A cache row that would exceed a unit's capacity is never
 *     written; the kernel records it in a sticky device word that ag_poll_error reports.
 *   - No C++ exception crosses this boundary.  An ag_ctx is not thread-safe; distinct contexts are.
 *   - The calls of one context share its workspace and a few arrival counters that are zero between launches:
 *     work enqueued through one context must not overlap on the device (use one stream, or order the streams
 *     with events); give work that is meant to run concurrently a context of its own.
 *   - Flags: uint8, 1 (any non-zero) = retain, 0 = evict, stored head-major [B, Hkv, L].
 *   - GQA: query head i reads KV head i / (Hq / Hkv); flags and caches are per KV head.
 *   - Supported: dtype bf16 with D = 128 or 64 (MFMA path) and fp32 with D <= 256 (plain-ALU path);
 *     H_f <= 32; Hq / Hkv in {1, 2, 4, 8}.
 */
#ifndef AG_H
#define AG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ag_ctx ag_ctx; /* opaque; owns only its workspace */

typedef enum {
  AG_OK = 0,
  AG_EINVAL = 1,       /* null pointer, non-positive size, Hq % Hkv != 0, tau outside (0,1), ...   */
  AG_EUNSUPPORTED = 2, /* shape or dtype outside the supported envelope                             */
  AG_ECAPACITY = 3,    /* a cache unit overflowed on the device (row dropped, nothing out of bounds) */
  AG_EWORKSPACE = 4,   /* the context's workspace is smaller than this call needs                   */
  AG_EHIP = 5          /* HIP runtime error, or a context without a device                          */
} ag_status;

typedef enum { AG_F32 = 0, AG_BF16 = 1 } ag_dtype;

/*
 * Gate settings of the paper's two experiments: threshold tau of Eq. 4 and the constant gamma that
 * Sec. 3.5 ("Initialization") adds inside the sigmoid.  gamma enters ag_gate as a bias of gamma in every head.
 * Continual pre-training (Sec. 4.1, training details): tau = 0.5, gamma = 2.
 * Supervised fine-tuning (Sec. 4.2, implementation details): tau = 0.3, gamma = 0.
 */
#define AG_TAU_PRETRAIN 0.5f
#define AG_GAMMA_PRETRAIN 2.0f
#define AG_TAU_FINETUNE 0.3f
#define AG_GAMMA_FINETUNE 0.0f

/*
 * Ragged per-(batch, KV head) cache.  Unit u = b * Hkv + g owns rows [row_off[u], row_off[u+1]) of k, v and
 * idx; its first len[u] rows are valid, in increasing token position.  All pointers are device memory.
 */
typedef struct {
  void *k;                /* [total_rows, D] rows in `dtype`                                   */
  void *v;                /* [total_rows, D]                                                   */
  int32_t *idx;           /* [total_rows]   token position of each cached row                  */
  const int64_t *row_off; /* [B*Hkv + 1]    first row of each unit (capacity = difference)     */
  int32_t *len;           /* [B*Hkv]        valid rows per unit; updated by compact and decode */
  int64_t total_rows;     /* host value: rows allocated in k, v, idx (= row_off[B*Hkv])        */
  int32_t B, Hkv, D;
  ag_dtype dtype;
} ag_kv_cache;

/*
 * Context.  ag_create binds to HIP device `device` and allocates `workspace_bytes` of device workspace
 * (ag_workspace_bytes gives a sufficient size).  device = -1 makes a context without a device: every call
 * still validates its arguments, then returns AG_EHIP instead of launching (used to test error paths on a
 * machine with no GPU).  ag_last_error returns a message for the last non-OK status of this context.
 */
ag_status ag_create(ag_ctx **out, int device, size_t workspace_bytes);
void ag_destroy(ag_ctx *ctx);
const char *ag_last_error(const ag_ctx *ctx);

/* Workspace that covers ag_gate (d_in features), ag_compact_kv, ag_prefill_attn (with cache == NULL, which
 * compacts into the workspace) and ag_decode_attn over caches of at most `cache_rows` rows in total. */
size_t ag_workspace_bytes(int B, int L, int Hq, int Hkv, int D, ag_dtype dtype, int d_in, int64_t cache_rows);

/* Synchronise `stream`, read and clear the sticky device error word.  AG_OK or AG_ECAPACITY.
 * (Kernel timing and machine probes for benchmarks are declared in ag_bench.h; they are no part of the method.) */
ag_status ag_poll_error(ag_ctx *ctx, void *hip_stream);

/*
 * Gate (Eq. 3 and Eq. 4; the constant inside the sigmoid is Sec. 3.5 "Initialization").
 *   logit[b,t,h] = sum_c feat[b,t,c] * w_gate[c,h] + bias[h]          (fp32 accumulate)
 *   flag [b,h,t] = Sigmoid(logit) > tau  <=>  logit > ln(tau/(1-tau))   (strict; compared in fp32)
 *   flag [b,h,t] = 1 for t < n_sink
 * feat [B, L, d_in] and w_gate [d_in, H_f] in `dtype`; bias fp32 [H_f].  feat is the hidden state for the
 * linear gate of Sec. 3.4, or the concatenated MHA' head outputs (d_in = h' * d'_k, w_gate = W^{O'}) for the
 * main architecture of Sec. 3.3.  logits_out fp32 [B, L, H_f] may be NULL; flags_out uint8 [B, H_f, L].
 * bf16 needs d_in % 64 == 0.
 */
ag_status ag_gate(ag_ctx *ctx, void *hip_stream, const void *feat, ag_dtype dtype, int B, int L, int d_in,
                  const void *w_gate, const float *bias, int H_f, float tau, int n_sink, float *logits_out,
                  uint8_t *flags_out);

/*
 * The gate fused with the normalisation that produces its input (the kernel fusion Sec. 4.2.3 leaves as future
 * work, for the linear gate of Sec. 3.4).  The paper's X (Eq. 3) is the attention block's input, which the decoder
 * models of Sec. 4 obtain from the residual stream h by a root-mean-square normalisation with weights g:
 *   x[b,t,c]     = (h[b,t,c] * r[b,t]) * g[c],  r = 1 / sqrt(mean_c h[b,t,c]^2 + eps)    (fp32, one rounding to bf16)
 *   logit, flag  = as ag_gate computes them from the stored x
 * in one pass over h: x_out is written for the projections that follow and the gate needs no second read of it.
 * h, x_out [B, L, d_in], norm_w [d_in] and w_gate [d_in, H_f] bf16, 16-byte aligned (w_gate only for speed);
 * x_out may be h itself (in-place normalisation).  bias fp32 [H_f]; logits_out fp32 [B, L, H_f] may be NULL;
 * flags_out uint8 [B, H_f, L].  Built for bf16, d_in % 64 == 0, d_in <= 8192, eps > 0 (else AG_EUNSUPPORTED /
 * AG_EINVAL).  Needs no more workspace than ag_gate on the same sizes.
 */
ag_status ag_rmsnorm_gate(ag_ctx *ctx, void *hip_stream, const void *h, ag_dtype dtype, int B, int L, int d_in,
                          const void *norm_w, float eps, const void *w_gate, const float *bias, int H_f, float tau,
                          int n_sink, void *x_out, float *logits_out, uint8_t *flags_out);

/*
 * The paper's main gate (Sec. 3.3, Eq. 3): a small multi-head attention MHA' over the hidden states, then the
 * gate's output projection and the threshold of Eq. 4.
 *   Q', K', V' = x w_qkv     x [B, L, d_model]; w_qkv [d_model, 3 * h_prime * d_prime], columns ordered
 *                            (Q' | K' | V'), inside each block head-major (head 0's d_prime columns first)
 *   A          = per head, causal softmax(Q' K'^T / sqrt(d_prime)) V' over the whole prompt (nothing is
 *                evicted inside the gate), stored in `dtype`
 *   logits     = concat_heads(A) w_o + bias     w_o [h_prime * d_prime, H_f], bias fp32 [H_f]
 *   flags      = logits > ln(tau / (1 - tau)); the first n_sink tokens forced to 1        (as ag_gate)
 * logits_out fp32 [B, L, H_f] (NULL allowed), flags_out uint8 [B, H_f, L].  Built for bf16 with d_prime = 128
 * (the paper's h' = 4, d'_k = 128), d_model % 64 == 0, H_f <= 32; anything else is AG_EUNSUPPORTED.  The
 * intermediates live in the workspace; ag_gate_mha_workspace_bytes gives a sufficient size (0 for shapes that
 * are not supported).
 */
size_t ag_gate_mha_workspace_bytes(int B, int L, int d_model, int h_prime, int d_prime, int H_f);
ag_status ag_gate_mha(ag_ctx *ctx, void *hip_stream, const void *x, ag_dtype dtype, int B, int L, int d_model,
                      const void *w_qkv, int h_prime, int d_prime, const void *w_o, const float *bias, int H_f,
                      float tau, int n_sink, float *logits_out, uint8_t *flags_out);

/*
 * Packed cache layout (Sec. 3.3: only the retained k, v take cache memory -- the saving that Sec. 4.2.3 and Fig. 3
 * report).  Computes, on the device and from the flags alone, slab offsets that give every unit exactly its
 * retained rows plus `room` spare rows for the tokens appended while decoding:
 *   row_off[0] = 0,   row_off[u + 1] = min(row_off[u] + kept(u) + room, total_rows),   kept(u) = #{t : flags[u,t] != 0}
 * so a cache of sum_u kept(u) + B * Hkv * room rows holds the prompt instead of B * Hkv * (L + room).  Call it before
 * ag_compact_kv, ag_compact_prefill_attn or ag_project_compact_kv on the same flags, with cache->row_off = row_off;
 * decoding then appends into the spare rows (a unit that has used them up drops further rows: ag_poll_error).
 * flags uint8 [B, Hkv, L]; row_off int64 [B * Hkv + 1], written; total_rows = rows allocated in the cache's k, v, idx
 * (host value): a layout that needs more is cut off there -- the units past the end get no rows, the compaction
 * drops theirs and ag_poll_error reports AG_ECAPACITY.  rows_needed (device int64, may be NULL) receives the rows
 * the layout would need, sum_u (kept(u) + room), so that a caller can size or check its allocation without
 * synchronising here.  Needs 4 * B * Hkv bytes of workspace.
 */
ag_status ag_pack_row_off(ag_ctx *ctx, void *hip_stream, const uint8_t *flags, int B, int Hkv, int L, int room,
                          int64_t total_rows, int64_t *row_off, int64_t *rows_needed);

/*
 * KV-cache after prefilling (Sec. 3.3; Sec. 3.1 prefilling stage): stable stream compaction.
 * For each unit, rows t of k, v [B, Hkv, L, D] with flags[b,g,t] != 0 are copied, in increasing t, to the
 * unit's cache rows; idx gets pos0 + t and len the number of rows.  The result is unique, hence bit-exact.
 * cache->row_off holds the units' slab offsets: filled by the caller (any layout, e.g. u * capacity) or by
 * ag_pack_row_off (packed: retained rows + room); rows beyond a unit's capacity are dropped (ag_poll_error).
 */
ag_status ag_compact_kv(ag_ctx *ctx, void *hip_stream, const void *k, const void *v, const uint8_t *flags,
                        int L, int pos0, ag_kv_cache *cache);

/*
 * Flag-masked causal attention (Eq. 2 with the mask of Eq. 5).  For query head i (KV head g = i / (Hq/Hkv))
 * and row j the visible keys are { t < j : flags[b,g,t] != 0 } plus j itself:
 *   out[b,i,j,:] = sum_t softmax_t(scale * q_j . k_t) v_t   over that set (fp32 accumulate).
 * q, out [B, Hq, L, D]; k, v [B, Hkv, L, D]; flags [B, Hkv, L].  `cache`, if not NULL, must be the result of
 * ag_compact_kv on the same k, v, flags with no overflow (the kernel attends over the compacted rows and
 * takes each row's own k_j, v_j from k, v); with NULL the call compacts into the workspace first.
 * Evicted keys contribute exactly zero, so a fully evicted head returns out[j] = v[j].
 */
ag_status ag_prefill_attn(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                          const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype,
                          float scale, const ag_kv_cache *cache, void *out);

/*
 * The same attention with a window of recent tokens that stay visible whatever their flag (Table 6 of the appendix, the
 * "keep recent tokens" settings): the visible keys of row j are
 *   { t < j : flags[b,g,t] != 0 }  plus  { t : j - n_recent < t <= j }.
 * n_recent = 1 is ag_prefill_attn (only the diagonal); 1 <= n_recent <= 64, else AG_EINVAL.  Arguments, layouts
 * and the meaning of `cache` are those of ag_prefill_attn; the evicted tokens inside the window are read from
 * k, v (they are not in the cache).
 */
ag_status ag_prefill_attn_recent(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                                 const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype,
                                 float scale, const ag_kv_cache *cache, int n_recent, void *out);

/*
 * The layer's own key/value projection (Eq. 2: K = X W^K, V = X W^V) fused with ag_compact_kv, for bf16 and head
 * size 128: the kept rows go from the projection's accumulators straight into the cache, so the compaction pass
 * and its second read of K and V disappear (the kernel fusion that Sec. 4.2.3, "Inference Efficiency", leaves
 * as future work).
 *   x      [B, L, d_model] bf16, d_model % 64 == 0
 *   w_kv   [d_model, 2 * Hkv * 128] bf16: the K columns of all heads (head h at columns 128 h ..), then the V columns
 *   flags  [B, Hkv, L]
 *   kv_out one allocation of two [B, Hkv, L, 128] bf16 tensors back to back, k then v: every token's own k, v, which
 *          the diagonal of Eq. 5 needs whether the token is kept or not (pass them to ag_prefill_attn as k, v)
 *   cache  as in ag_compact_kv (B, Hkv from the cache; D = 128, bf16; row_off filled by the caller): receives the
 *          kept rows, idx = pos0 + t and len; rows beyond a unit's capacity are dropped (ag_poll_error)
 * The cache rows are bit-identical to the rows of kv_out they copy.  AG_EUNSUPPORTED for other dtypes or sizes.
 */
size_t ag_project_compact_workspace_bytes(int B, int L, int Hkv);
ag_status ag_project_compact_kv(ag_ctx *ctx, void *hip_stream, const void *x, ag_dtype dtype, int B, int L,
                                int d_model, const void *w_kv, const uint8_t *flags, int pos0, void *kv_out,
                                ag_kv_cache *cache);

/*
 * ag_compact_kv followed by ag_prefill_attn_recent on the same k, v, flags, as one call that scans the flags once:
 * `cache` (row_off filled by the caller) receives the compacted rows, idx (pos0 + t) and len exactly as from
 * ag_compact_kv, and out the attention over them.  The prefilling stage of one layer (Sec. 3.1, Sec. 3.3).
 */
ag_status ag_compact_prefill_attn(ag_ctx *ctx, void *hip_stream, const void *q, const void *k, const void *v,
                                  const uint8_t *flags, int B, int L, int Hq, int Hkv, int D, ag_dtype dtype,
                                  float scale, int pos0, ag_kv_cache *cache, int n_recent, void *out);

/*
 * One decoding step (Sec. 3.1 decoding stage; the gate is not run during decoding, Sec. 3.4).
 * For every (b, query head i): keys = cache rows of unit (b, g) followed by k_new[b,g]; same for values;
 * out[b,i,:] = softmax-weighted sum (the new token always attends to itself, Eq. 5 diagonal; an empty cache
 * returns v_new).  Then, for every unit with new_flags == NULL or new_flags[b,g] != 0, (k_new, v_new, pos) is
 * appended and len incremented.  All query heads of a group read the cache before the append.
 * q, out [B, Hq, D]; k_new, v_new [B, Hkv, D] in cache->dtype; new_flags uint8 [B, Hkv] or NULL.
 */
ag_status ag_decode_attn(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                         const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache, void *out);

/*
 * ag_decode_attn for callers that cannot allocate device memory or be handed a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same
 * results as ag_decode_attn, but the per-item records that the two decode kernels exchange live in a static
 * device array of the library (ag_decode_static_scratch_bytes() = 16 MiB per GPU, held until the process ends)
 * instead of the context's workspace; the call allocates and frees nothing and a context made with
 * workspace_bytes = 0 is enough.  The array's device address is looked up once per GPU inside ag_create.
 * A cache needs ag_decode_scratch_bytes(cache, Hq) bytes (about 4 (D + 2) (Hq / Hkv) bytes per 128 cache rows
 * of total_rows, plus as much per unit); a cache that needs more than the array holds is rejected with
 * AG_EWORKSPACE and nothing is launched.  Nothing in the array has to be zero between calls.  Every call on one
 * GPU shares that GPU's array, whatever its context: two such calls that overlap on the device race; keep them on
 * one stream or order them with events.
 */
size_t ag_decode_static_scratch_bytes(void);
size_t ag_decode_scratch_bytes(const ag_kv_cache *cache, int Hq);
ag_status ag_decode_attn_static(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                                const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache,
                                void *out);

/*
 * Decoding with the recent-token window (Table 6 of the appendix, "keep recent tokens"): the tokens at the n_recent - 1 positions
 * before the new one stay visible whatever their flag.  The evicted ones are not in the cache, so the last
 * n_recent tokens of every unit live in a small ring, slot = position % n_recent (caller-owned device memory):
 *   k, v   [B*Hkv, n_recent, D] in the cache's dtype;  flags uint8 [B*Hkv, n_recent] (keep flag of the token in
 *   the slot);  pos int32 [B*Hkv, n_recent] (its position; a large negative number marks an empty slot).
 * ag_recent_fill loads the ring with the last min(L, n_recent) prompt tokens (k, v [B, Hkv, L, D], flags
 * [B, Hkv, L], first token at position pos0) and marks the other slots empty; call it once after prefilling.
 * ag_decode_attn_recent is ag_decode_attn plus: every ring token t with pos - n_recent < t < pos and flag 0 is one
 * more key/value (those with flag 1 are cache rows already); afterwards the new token (with its flag) takes slot
 * pos % n_recent.  `pos` must advance by one per step.  ring == NULL is ag_decode_attn.  2 <= n_recent <= 64.
 */
typedef struct {
  void *k, *v;
  uint8_t *flags;
  int32_t *pos;
  int32_t n_recent;
} ag_recent_ring;

ag_status ag_recent_fill(ag_ctx *ctx, void *hip_stream, const void *k, const void *v, const uint8_t *flags, int B,
                         int L, int Hkv, int D, ag_dtype dtype, int pos0, ag_recent_ring *ring);
ag_status ag_decode_attn_recent(ag_ctx *ctx, void *hip_stream, const void *q, const void *k_new, const void *v_new,
                                const uint8_t *new_flags, int pos, int Hq, float scale, ag_kv_cache *cache,
                                ag_recent_ring *ring, void *out);

#ifdef __cplusplus
}
#endif
#endif /* AG_H */
