// Machine probes used by the benchmark to state what this GPU actually sustains: a dense bf16 MFMA loop with
// no memory traffic and a streaming copy through HBM.  They put the roofline fractions next to measured peaks
// as well as the data-sheet ones.  Not part of the attention path.
#include "ag_internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__global__ __launch_bounds__(256) void ag_probe_mfma_kernel(int iters, float *sink) {
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
    b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 12345.678f) sink[0] = s;  // keeps the loop alive; practically never true
}

// The same loop on operands that change from one MFMA to the next and look like data: eight A and eight B fragments
// per lane with pseudo-random signs, mantissas and exponents (values of magnitude 1/4 .. 4), cycled so that
// consecutive MFMAs of the matrix pipe never see the same inputs.  The power an MFMA draws depends on how many
// bits toggle, so this is the ceiling that applies to a kernel working on real activations.  idle > 0: after every
// 8 MFMAs the wave sleeps idle x 64 cycles, which sets the matrix pipe's duty cycle when one wave runs per SIMD
// (256 busy cycles per group): the chip then clocks higher, and the pair (duty, rate) shows how the power budget
// trades clock against activity.
__global__ __launch_bounds__(256) void ag_probe_mfma_data_kernel(int iters, float *sink, int idle) {
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  uint4 a[8], b[8];
  uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
  auto next = [&]() {  // two bf16 with random sign and mantissa, exponent 125..128
    h = h * 1664525u + 1013904223u;
    const uint32_t lo = (h & 0x807fu) | ((125u + ((h >> 8) & 3u)) << 7);
    const uint32_t hi = ((h >> 16) & 0x807fu) | ((125u + ((h >> 24) & 3u)) << 7);
    return lo | (hi << 16);
  };
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = make_uint4(next(), next(), next(), next());
    b[j] = make_uint4(next(), next(), next(), next());
  }
  for (int it = 0; it < iters; it += 2) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[j]),
                                                           __builtin_bit_cast(bf16x8, b[(j * 3 + 1) & 7]), acc[j & 3], 0, 0, 0);
    for (int p = 0; p < idle; ++p) __builtin_amdgcn_s_sleep(1);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 12345.678f) sink[0] = s;
}

__global__ __launch_bounds__(256) void ag_probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                            size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" {

static ag_status probe_mfma(ag_ctx *ctx, void *hip_stream, int iters, bool data, int idle, double *tflops);

ag_status ag_probe_mfma(ag_ctx *ctx, void *hip_stream, int iters, double *tflops) {
  return probe_mfma(ctx, hip_stream, iters, false, -1, tflops);
}

ag_status ag_probe_mfma_data(ag_ctx *ctx, void *hip_stream, int iters, double *tflops) {
  return probe_mfma(ctx, hip_stream, iters, true, -1, tflops);
}

ag_status ag_probe_mfma_duty(ag_ctx *ctx, void *hip_stream, int iters, int idle, double *tflops) {
  if (idle < 0 || idle > 64) return AG_EINVAL;
  return probe_mfma(ctx, hip_stream, iters, true, idle, tflops);
}

// idle < 0: two workgroups per CU (2 waves per SIMD), no pauses; idle >= 0: one per CU with idle x 64-cycle pauses
static ag_status probe_mfma(ag_ctx *ctx, void *hip_stream, int iters, bool data, int idle, double *tflops) {
  if (!ctx || !tflops || iters <= 0) return AG_EINVAL;
  iters = (iters + 1) & ~1;
  if (ctx->device < 0) return ag_fail(ctx, AG_EHIP, "context has no device");
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipSetDevice(ctx->device) != hipSuccess || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return ag_fail(ctx, AG_EHIP, "ag_probe_mfma: event creation failed");
  const int blocks = ctx->num_cu * (idle < 0 ? 2 : 1);  // 8 waves per CU, 2 per SIMD; or 4, 1 per SIMD
  float *sink = reinterpret_cast<float *>(ctx->d_err) + 8;
  const int pauses = idle < 0 ? 0 : idle;
  auto launch = [&](int n) {
    if (data) hipLaunchKernelGGL(ag_probe_mfma_data_kernel, dim3(blocks), dim3(256), 0, s, n, sink, pauses);
    else hipLaunchKernelGGL(ag_probe_mfma_kernel, dim3(blocks), dim3(256), 0, s, n, sink);
  };
  launch((iters / 8 + 2) & ~1);  // warm-up
  (void)hipEventRecord(e0, s);
  launch(iters);
  (void)hipEventRecord(e1, s);
  float ms = 0.f;
  hipError_t e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return ag_fail(ctx, AG_EHIP, "ag_probe_mfma: %s", hipGetErrorString(e));
  const double flops = (double)blocks * 4 /*waves*/ * iters * 4 /*mfma*/ * (2.0 * 32 * 32 * 16);
  *tflops = flops / (ms * 1e-3) / 1e12;
  return AG_OK;
}

ag_status ag_probe_copy(ag_ctx *ctx, void *hip_stream, size_t bytes, double *gbs) {
  if (!ctx || !gbs || bytes < 4096) return AG_EINVAL;
  if (ctx->device < 0) return ag_fail(ctx, AG_EHIP, "context has no device");
  bytes &= ~(size_t)255;
  if (2 * bytes > ctx->ws_bytes) return ag_fail(ctx, AG_EWORKSPACE, "ag_probe_copy: needs a workspace of 2 x %zu bytes", bytes);
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipSetDevice(ctx->device) != hipSuccess || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return ag_fail(ctx, AG_EHIP, "ag_probe_copy: event creation failed");
  const uint4 *src = reinterpret_cast<const uint4 *>(ctx->ws);
  uint4 *dst = reinterpret_cast<uint4 *>(ctx->ws + bytes);
  const size_t n = bytes / 16;
  const int blocks = ctx->num_cu * 8;
  hipLaunchKernelGGL(ag_probe_copy_kernel, dim3(blocks), dim3(256), 0, s, src, dst, n);  // warm-up
  (void)hipEventRecord(e0, s);
  for (int r = 0; r < 4; ++r) hipLaunchKernelGGL(ag_probe_copy_kernel, dim3(blocks), dim3(256), 0, s, src, dst, n);
  (void)hipEventRecord(e1, s);
  float ms = 0.f;
  hipError_t e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return ag_fail(ctx, AG_EHIP, "ag_probe_copy: %s", hipGetErrorString(e));
  *gbs = 4.0 * 2.0 * (double)bytes / (ms * 1e-3) / 1e9;  // read + write
  return AG_OK;
}

}  // extern "C"
