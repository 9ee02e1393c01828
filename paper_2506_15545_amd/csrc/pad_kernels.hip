// Row padding for sequence lengths that are not a multiple of the matrix-core kernels' 128-row tiles: the layer is
// causal, so rows appended after the last token change nothing before them, and zero rows of dO contribute nothing
// to any gradient.  Tensors are [B, T, H*D]; the padded copy is [B, Tp, H*D] with zero rows t >= T.
#include "common.hpp"
#include "kernels.hpp"

namespace rattn {

namespace {

// one thread per 16 bytes of the destination
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int B, int T,
                                                       int Tp, long long row_vecs) {
  const long long total = (long long)B * Tp * row_vecs;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long c = i % row_vecs, r = i / row_vecs;
    const int t = (int)(r % Tp), b = (int)(r / Tp);
    dst[i] = t < T ? src[((long long)b * T + t) * row_vecs + c] : make_uint4(0u, 0u, 0u, 0u);
  }
}

// one thread per 16 bytes of the destination (the unpadded tensor)
__global__ __launch_bounds__(256) void unpad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int B,
                                                         int T, int Tp, long long row_vecs) {
  const long long total = (long long)B * T * row_vecs;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long c = i % row_vecs, r = i / row_vecs;
    const int t = (int)(r % T), b = (int)(r / T);
    dst[i] = src[((long long)b * Tp + t) * row_vecs + c];
  }
}

int blocks_for(long long total) {
  const long long n = (total + 255) / 256;
  return (int)(n < 16384 ? (n > 0 ? n : 1) : 16384);
}

}  // namespace

void pad_rows(const void* src, void* dst, int B, int T, int Tp, size_t row_bytes, hipStream_t st) {
  const long long rv = (long long)(row_bytes / 16);
  ProfScope ps("pad_rows_kernel", st);
  pad_rows_kernel<<<blocks_for((long long)B * Tp * rv), 256, 0, st>>>((const uint4*)src, (uint4*)dst, B, T, Tp, rv);
}

void unpad_rows(const void* src, void* dst, int B, int T, int Tp, size_t row_bytes, hipStream_t st) {
  const long long rv = (long long)(row_bytes / 16);
  ProfScope ps("unpad_rows_kernel", st);
  unpad_rows_kernel<<<blocks_for((long long)B * T * rv), 256, 0, st>>>((const uint4*)src, (uint4*)dst, B, T, Tp, rv);
}

}  // namespace rattn
