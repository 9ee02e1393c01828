// Machine probe used by the benchmark: what a loop of nothing but matrix-core instructions sustains on this
// device, as the context for the fractions of the published peak that the benchmark reports.
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"

namespace rattn {

namespace {

// 16 * iters v_mfma_f32_32x32x16_bf16 per wave, on four independent accumulators.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* sink, int iters) {
  const int lane = lane_id();
  bf16x8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.001f * (lane + i)); b[i] = (__bf16)(0.002f * (lane - i)); }
  f32x16_t acc[4] = {{0}, {0}, {0}, {0}};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = mfma32(a, b, acc[j]);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  if (s == 1.2345f) sink[0] = s;  // keeps the loop alive; practically never true
}

}  // namespace

double probe_mfma(float* sink, int iters, int blocks, hipStream_t st) {
  probe_mfma_kernel<<<blocks, 256, 0, st>>>(sink, iters);
  return 2.0 * 32 * 32 * 16 * 16.0 * iters * 4.0 * blocks;  // FLOPs issued
}

}  // namespace rattn
