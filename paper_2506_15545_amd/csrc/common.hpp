// Shared device helpers for librattn (gfx950 only: 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "kernels.hpp"

namespace rattn {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename IO> struct io_traits;

template <> struct io_traits<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
  // 8 consecutive elements, p 16-byte aligned
  static __device__ __forceinline__ void ld8(const float* p, float (&o)[8]) {
    float4 a = *reinterpret_cast<const float4*>(p);
    float4 b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
};

template <> struct io_traits<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ void ld8(const bf16_t* p, float (&o)[8]) {
    uint4 r = *reinterpret_cast<const uint4*>(p);
    o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
// value held by lane `l` (wave-uniform l) broadcast to the whole wave through an SGPR
__device__ __forceinline__ float bcast(float x, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}
// Feature map of the linear branch: softmax over the features (Sec. 3.1), or the ablation's ReLU / identity
// (Sec. 4.5).  Every map is written phi(x)[f] = feat(x[f], m) / z with row statistics (m, z): the row maximum and
// the sum of exponentials for softmax, (0, 1) for the other two.  `phi` is uniform over a launch.
__device__ __forceinline__ float feat(float x, float m, int phi) {
  if (phi == PHI_SOFTMAX) return expf(x - m);
  return phi == PHI_RELU ? fmaxf(x, 0.f) : x;
}
// d/dx of sum_f phi(x)[f] df[f] for one element: x the input, f = phi(x)[f], inner = <df, phi(x)> (softmax only)
__device__ __forceinline__ float feat_bwd(float x, float f, float df, float inner, int phi) {
  if (phi == PHI_SOFTMAX) return f * (df - inner);
  return (phi == PHI_IDENTITY || x > 0.f) ? df : 0.f;
}
// phi of a row of 64*EPL features spread over the wave (element d in lane d % 64, register d / 64)
template <int EPL>
__device__ __forceinline__ void feature_row(const float (&x)[EPL], float (&f)[EPL], int phi) {
  if (phi == PHI_SOFTMAX) {
    float m = x[0];
#pragma unroll
    for (int e = 1; e < EPL; ++e) m = fmaxf(m, x[e]);
    m = wave_max(m);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) { f[e] = expf(x[e] - m); s += f[e]; }
    s = 1.f / wave_sum(s);
#pragma unroll
    for (int e = 0; e < EPL; ++e) f[e] *= s;
  } else {
#pragma unroll
    for (int e = 0; e < EPL; ++e) f[e] = phi == PHI_RELU ? fmaxf(x[e], 0.f) : x[e];
  }
}
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

}  // namespace rattn
