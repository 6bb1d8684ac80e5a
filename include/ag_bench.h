/*
 * libag -- instrumentation for benchmarks: per-kernel timing and two machine probes.  No part of the Attention-Gate
 * path (that is ag.h); exported by the same library so that a benchmark can time the kernels the path launches.
 */
#ifndef AG_BENCH_H
#define AG_BENCH_H

#include "ag.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel timing for benchmarks.  While enabled, every kernel the library launches carries a pair of HIP events
 * on the call's stream: the main kernels (fused gate, scan + compaction, prefill, decode partial and merge,
 * projection) have them attached to the launch itself, so the duration is the kernel's own; the remaining
 * launches are bracketed by records on the stream.  Up to 1024 launches per kernel id are remembered; later
 * ones are not timed.  Leave timing off while the stream is being captured into a HIP graph.
 * ag_timing_enable(ctx, 1) resets the counts; ag_timing_read waits for the recorded events and returns the summed
 * duration and the number of launches of one kernel id in [0, ag_timing_kernels()).
 * Ids: 0 gate (GEMM), 1 gate_finalize, 2 flag_scan, 3 compact, 4 prefill, 5 decode_partial, 6 decode_merge,
 * 7 mha_proj, 8 mha_attn, 9 norm_gate; ag_timing_kernel_name gives the names.
 */
int ag_timing_kernels(void);
const char *ag_timing_kernel_name(int kernel_id);
ag_status ag_timing_enable(ag_ctx *ctx, int on);
ag_status ag_timing_read(ag_ctx *ctx, int kernel_id, double *total_ms, int *launches);

/*
 * Machine probes for benchmarks (no part of the attention path).  ag_probe_mfma runs a register-only loop of
 * `iters` x 4 v_mfma_f32_32x32x16_bf16 per wave on 8 waves per CU and returns the sustained TFLOP/s;
 * ag_probe_copy streams `bytes` (>= 4096) from one half of the context's workspace to the other, four times,
 * and returns read+write GB/s.  Both synchronise on their own events.
 */
ag_status ag_probe_mfma(ag_ctx *ctx, void *hip_stream, int iters, double *tflops);
/* The same loop on operands that look like data (pseudo-random signs, mantissas and exponents, different from one
 * MFMA to the next): an MFMA's power depends on how many bits toggle, and under the board's power cap that decides
 * the clock.  This is the ceiling that applies to a kernel working on real activations. */
ag_status ag_probe_mfma_data(ag_ctx *ctx, void *hip_stream, int iters, double *tflops);
/* The data-operand loop with ONE wave per SIMD (4 per CU) that sleeps `idle` x 64 cycles (0 <= idle <= 64) after
 * every 8 MFMAs, i.e. with the matrix pipe busy 256 / (256 + 64 idle) of the time and nothing else running.  The
 * rate at a given duty cycle, compared with duty x (rate at idle = 0), shows how far the chip raises its clock when
 * the pipe is busy less often: what a kernel at that duty cycle could reach if its other work cost no power. */
ag_status ag_probe_mfma_duty(ag_ctx *ctx, void *hip_stream, int iters, int idle, double *tflops);
ag_status ag_probe_copy(ag_ctx *ctx, void *hip_stream, size_t bytes, double *gbs);

#ifdef __cplusplus
}
#endif
#endif /* AG_BENCH_H */
