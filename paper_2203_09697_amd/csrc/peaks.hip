// Measurement aid (not a step of the method): achievable rates of this GPU, measured with the
// simplest kernels that can reach them, so that a kernel's roofline fraction can be quoted against
// the measured rate as well as against the published one.
//   copy:  16-byte loads and stores of a large buffer (bytes read + bytes written per second)
//   mfma:  a register-resident chain of independent matrix-core instructions, no memory traffic
#include <stdarg.h>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ void __launch_bounds__(256)
peak_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

constexpr int MFMA_CHAINS = 4;     // independent accumulators per wavefront
constexpr int MFMA_ITERS = 2048;   // instructions per chain

__global__ void __launch_bounds__(256)
peak_mfma_f32_kernel(float* __restrict__ sink) {
  f32x16 acc[MFMA_CHAINS];
#pragma unroll
  for (int c = 0; c < MFMA_CHAINS; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
  const float a = 1.0f + (float)(threadIdx.x & 7) * 0.125f, b = 0.5f;
  for (int it = 0; it < MFMA_ITERS; ++it)
#pragma unroll
    for (int c = 0; c < MFMA_CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < MFMA_CHAINS; ++c) s += acc[c][0] + acc[c][15];
  if (s == 12345.678f) sink[0] = s;   // keeps the chain alive; never true in practice
}

__global__ void __launch_bounds__(256)
peak_mfma_bf16_kernel(float* __restrict__ sink) {
  f32x16 acc[MFMA_CHAINS];
#pragma unroll
  for (int c = 0; c < MFMA_CHAINS; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(1.0f + (float)((threadIdx.x + i) & 7) * 0.125f);
    b[i] = (__bf16)0.5f;
  }
  for (int it = 0; it < MFMA_ITERS; ++it)
#pragma unroll
    for (int c = 0; c < MFMA_CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < MFMA_CHAINS; ++c) s += acc[c][0] + acc[c][15];
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace

extern "C" {

int gp_measure_peaks(gp_ctx* ctx, void* ws, size_t ws_bytes, double* copy_gbps, double* mfma_f32_tflops,
                     double* mfma_bf16_tflops) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, ws && copy_gbps && mfma_f32_tflops && mfma_bf16_tflops, "gp_measure_peaks: NULL pointer");
  GP_REQUIRE(ctx, ws_bytes >= (size_t)64 << 20, "gp_measure_peaks: workspace below 64 MiB");
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  hipEvent_t t0, t1;
  GP_HIP(ctx, hipEventCreate(&t0));
  GP_HIP(ctx, hipEventCreate(&t1));
  const size_t half = (ws_bytes / 2) & ~(size_t)255;
  const int64_t n16 = (int64_t)(half / 16);
  float* src = static_cast<float*>(ws);
  float* dst = reinterpret_cast<float*>(static_cast<char*>(ws) + half);
  const int reps = 10;
  float ms = 0.f;
  int rc = GP_OK;
  auto timed = [&](auto launch) -> int {
    launch();   // warm-up
    if (hipEventRecord(t0, st) != hipSuccess) return GP_HIP_ERROR;
    for (int r = 0; r < reps; ++r) launch();
    if (hipEventRecord(t1, st) != hipSuccess || hipEventSynchronize(t1) != hipSuccess ||
        hipEventElapsedTime(&ms, t0, t1) != hipSuccess || hipGetLastError() != hipSuccess)
      return GP_HIP_ERROR;
    return GP_OK;
  };
  if (gp_zero_async(st, ws, half) != (int)hipSuccess) rc = GP_HIP_ERROR;
  if (rc == GP_OK) rc = timed([&] { peak_copy_kernel<<<256 * 16, 256, 0, st>>>((const f32x4*)src, (f32x4*)dst, n16); });
  if (rc == GP_OK) *copy_gbps = 2.0 * (double)half * reps / (ms * 1e-3) / 1e9;
  const int blocks = 256 * 8;   // 8 workgroups of 4 wavefronts per CU
  const double inst = (double)blocks * 4 * MFMA_CHAINS * MFMA_ITERS * reps;
  if (rc == GP_OK) rc = timed([&] { peak_mfma_f32_kernel<<<blocks, 256, 0, st>>>(dst); });
  if (rc == GP_OK) *mfma_f32_tflops = inst * (2.0 * 32 * 32 * 2) / (ms * 1e-3) / 1e12;
  if (rc == GP_OK) rc = timed([&] { peak_mfma_bf16_kernel<<<blocks, 256, 0, st>>>(dst); });
  if (rc == GP_OK) *mfma_bf16_tflops = inst * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  if (rc != GP_OK) return gp_fail(ctx, rc, "gp_measure_peaks: a HIP call failed");
  return GP_OK;
}

}  // extern "C"
