// Zero-padded copies for shapes that the matrix-core kernels do not take directly:
//  * sequence lengths that are not a multiple of their 128-row tiles: the layer is causal, so rows appended after the
//    last token change nothing before them, and zero rows of dO contribute nothing to any gradient;
//  * a head size of 64: rows are widened to 128 features with zeros, which add nothing to any dot product; the
//    kernels are told that only 64 features carry data (RMS norms, softmax feature map).
// Tensors are [B, T, H, D]; the padded copy is [B, Tp, H, Dp] with zeros at t >= T and in features >= D.
// With D = 128 only the last, partial tile of every sequence is copied (tail buffers, see RaggedTails); the kernels
// address everything in front of it in place.
#include "common.hpp"
#include "kernels.hpp"

namespace rattn {

namespace {

// one thread per 16 bytes of the destination; hv / hvp = 16-byte vectors per head row in the source / destination
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int B, int T,
                                                       int Tp, int H, int hv, int hvp) {
  const long long total = (long long)B * Tp * H * hvp;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int c = (int)(i % hvp);
    long long r = i / hvp;
    const int h = (int)(r % H); r /= H;
    const int t = (int)(r % Tp), b = (int)(r / Tp);
    dst[i] = (t < T && c < hv) ? src[(((long long)b * T + t) * H + h) * hv + c] : make_uint4(0u, 0u, 0u, 0u);
  }
}

// one thread per 16 bytes of the destination (the unpadded tensor)
__global__ __launch_bounds__(256) void unpad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int B,
                                                         int T, int Tp, int H, int hv, int hvp) {
  const long long total = (long long)B * T * H * hv;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int c = (int)(i % hv);
    long long r = i / hv;
    const int h = (int)(r % H); r /= H;
    const int t = (int)(r % T), b = (int)(r / T);
    dst[i] = src[(((long long)b * Tp + t) * H + h) * hvp + c];
  }
}

struct TailSet {
  const uint4* src[4];
  uint4* dst[4];
  int H[4];
};

// blockIdx.y = tensor; one thread per 16 bytes of a [B,128,H,16 vectors] tail buffer.  GATHER: buffer <- rows
// Tfull + r of the [B,T,H,128] bf16 tensor, zero where Tfull + r >= T; else tensor rows < T <- buffer.
template <bool GATHER>
__global__ __launch_bounds__(256) void tail_rows_kernel(TailSet s, int B, int T, int Tfull) {
  const int i = blockIdx.y, H = s.H[i];
  const long long total = (long long)B * 128 * H * 16;
  for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
    const int c = (int)(e & 15);
    long long r = e >> 4;
    const int h = (int)(r % H); r /= H;
    const int row = (int)(r & 127), b = (int)(r >> 7);
    const bool live = Tfull + row < T;
    const long long full = (((long long)b * T + Tfull + row) * H + h) * 16 + c;
    if (GATHER) s.dst[i][e] = live ? s.src[i][full] : make_uint4(0u, 0u, 0u, 0u);
    else if (live) s.dst[i][full] = s.src[i][e];
  }
}

int blocks_for(long long total) {
  const long long n = (total + 255) / 256;
  return (int)(n < 16384 ? (n > 0 ? n : 1) : 16384);
}

}  // namespace

void pad_rows(const void* src, void* dst, int B, int T, int Tp, int H, size_t head_bytes, size_t head_bytes_padded,
              hipStream_t st) {
  const int hv = (int)(head_bytes / 16), hvp = (int)(head_bytes_padded / 16);
  ProfScope ps("pad_rows_kernel", st);
  pad_rows_kernel<<<blocks_for((long long)B * Tp * H * hvp), 256, 0, st>>>((const uint4*)src, (uint4*)dst, B, T, Tp, H, hv, hvp);
}

void unpad_rows(const void* src, void* dst, int B, int T, int Tp, int H, size_t head_bytes, size_t head_bytes_padded,
                hipStream_t st) {
  const int hv = (int)(head_bytes / 16), hvp = (int)(head_bytes_padded / 16);
  ProfScope ps("unpad_rows_kernel", st);
  unpad_rows_kernel<<<blocks_for((long long)B * T * H * hv), 256, 0, st>>>((const uint4*)src, (uint4*)dst, B, T, Tp, H, hv, hvp);
}

void gather_tails(int n, const void* const* src, void* const* tail, const int* H, int B, int T, hipStream_t st) {
  TailSet s = {};
  int Hmax = 1;
  for (int i = 0; i < n && i < 4; ++i) { s.src[i] = (const uint4*)src[i]; s.dst[i] = (uint4*)tail[i]; s.H[i] = H[i]; Hmax = H[i] > Hmax ? H[i] : Hmax; }
  ProfScope ps("tail_rows_kernel(gather)", st);
  tail_rows_kernel<true><<<dim3(blocks_for((long long)B * 128 * Hmax * 16), n), 256, 0, st>>>(s, B, T, T / 128 * 128);
}

void scatter_tails(int n, const void* const* tail, void* const* dst, const int* H, int B, int T, hipStream_t st) {
  TailSet s = {};
  int Hmax = 1;
  for (int i = 0; i < n && i < 4; ++i) { s.src[i] = (const uint4*)tail[i]; s.dst[i] = (uint4*)dst[i]; s.H[i] = H[i]; Hmax = H[i] > Hmax ? H[i] : Hmax; }
  ProfScope ps("tail_rows_kernel(scatter)", st);
  tail_rows_kernel<false><<<dim3(blocks_for((long long)B * 128 * Hmax * 16), n), 256, 0, st>>>(s, B, T, T / 128 * 128);
}

}  // namespace rattn
