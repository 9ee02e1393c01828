// Prefill -> decode hand-over: from the keys and values of a prompt of T tokens, the rings and the lagged
// linear-attention state a decode step at pos = T reads (Sec. 2.1: the last W keys/values; Sec. 2.2 / Eq. 4: the
// state sum_{s < T-W} phi(k_s)^T v_s).  A one-off per prompt, written for any shape the library accepts: plain
// fp32 vector arithmetic, keys split into segments whose partial states are summed in a fixed order.
#include "common.hpp"
#include "kernels.hpp"

namespace rattn {

namespace {

// ring slot (tok0 + s) % W <- row s of k / v for the last min(T, W) rows (row s is token tok0 + s of its sequence).
// One thread per 16 bytes.
__global__ __launch_bounds__(256) void export_ring_kernel(const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                          uint4* __restrict__ k_ring, uint4* __restrict__ v_ring,
                                                          int B, int T, int Hkv, int W, int row_vecs, int tok0) {
  const int first = max(0, T - W), ntok = T - first;
  const long long total = (long long)B * ntok * Hkv * row_vecs;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int c = (int)(i % row_vecs);
    long long r = i / row_vecs;
    const int g = (int)(r % Hkv); r /= Hkv;
    const int s = first + (int)(r % ntok);
    const int b = (int)(r / ntok);
    const size_t src = ((size_t)(b * T + s) * Hkv + g) * row_vecs + c;
    const size_t dst = (((size_t)b * Hkv + g) * W + (tok0 + s) % W) * row_vecs + c;
    k_ring[dst] = k[src];
    v_ring[dst] = v[src];
  }
}

// Partial state of one key segment.  grid (nseg, Hkv, B), 256 threads.  Keys are staged KB at a time: LPR lanes
// per key row compute phi (row softmax, or the ablation's ReLU / identity) into LDS, then every thread adds KB rank-one terms to the NR x 4 state
// entries it owns (rows rg + RG*j, columns 4*cg .. 4*cg+3).
template <typename IO, int D>
__global__ __launch_bounds__(256) void export_state_partial_kernel(const IO* __restrict__ k, const IO* __restrict__ v,
                                                                   float* __restrict__ partial, int T, int Hkv,
                                                                   int Tp, int seg_len, int phi) {
  constexpr int LPR = D / 8, KB = 256 / LPR;
  constexpr int CG = D / 4, RG = 256 / CG, NR = D / RG;
  __shared__ float kf[KB][D];
  __shared__ __align__(16) float vs[KB][D];
  const int seg = blockIdx.x, g = blockIdx.y, b = blockIdx.z, nseg = gridDim.x;
  const int tid = threadIdx.x;
  const int lo = seg * seg_len, hi = min(lo + seg_len, Tp);
  const int kr = tid / LPR, li = tid % LPR;
  const int cg = tid % CG, rg = tid / CG;
  float4 acc[NR];
#pragma unroll
  for (int j = 0; j < NR; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = lo; s0 < hi; s0 += KB) {
    const int s = s0 + kr;
    float x[8], y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { x[e] = -INFINITY; y[e] = 0.f; }
    if (s < hi) {
      const size_t off = ((size_t)(b * T + s) * Hkv + g) * D + 8 * li;
      io_traits<IO>::ld8(k + off, x);
      io_traits<IO>::ld8(v + off, y);
    }
    float m = x[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) m = fmaxf(m, x[e]);
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { x[e] = s < hi ? feat(x[e], m, phi) : 0.f; sum += x[e]; }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const float inv = s < hi ? (phi == PHI_SOFTMAX ? 1.f / sum : 1.f) : 0.f;
    __syncthreads();  // the previous batch has been consumed
#pragma unroll
    for (int e = 0; e < 8; ++e) { kf[kr][8 * li + e] = x[e] * inv; vs[kr][8 * li + e] = y[e]; }
    __syncthreads();
    for (int kk = 0; kk < KB; ++kk) {
      const float4 vv = *reinterpret_cast<const float4*>(&vs[kk][4 * cg]);
#pragma unroll
      for (int j = 0; j < NR; ++j) {
        const float f = kf[kk][rg + RG * j];
        acc[j].x += f * vv.x; acc[j].y += f * vv.y; acc[j].z += f * vv.z; acc[j].w += f * vv.w;
      }
    }
  }
  float4* out = reinterpret_cast<float4*>(partial + (((size_t)b * Hkv + g) * nseg + seg) * D * D);
#pragma unroll
  for (int j = 0; j < NR; ++j) out[(size_t)(rg + RG * j) * CG + cg] = acc[j];
}

// state[b,g] = (accumulate ? state[b,g] : 0) + sum over segments, in segment order.  One thread per float4.
__global__ __launch_bounds__(256) void export_state_reduce_kernel(const float4* __restrict__ partial, float4* state,
                                                                  int nseg, int vecs, long long total, int accumulate) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const long long bg = i / vecs, e = i % vecs;
  float4 s = accumulate ? state[i] : make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c = 0; c < nseg; ++c) {
    const float4 p = partial[(bg * nseg + c) * vecs + e];
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  state[i] = s;
}

}  // namespace

void prefill_export(const LayerDims& dm, int dtype, const void* k, const void* v, void* k_ring, void* v_ring,
                    float* state, float* partial, hipStream_t st, int tok0, bool accumulate) {
  const ExportPlan pl = export_plan(dm);
  const int esize = dtype == 0 ? 4 : 2;
  const int row_vecs = dm.D * esize / 16;
  {
    const long long total = (long long)dm.B * (dm.T < dm.W ? dm.T : dm.W) * dm.Hkv * row_vecs;
    const int blocks = (int)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
    ProfScope ps("export_ring_kernel", st);
    export_ring_kernel<<<blocks, 256, 0, st>>>((const uint4*)k, (const uint4*)v, (uint4*)k_ring, (uint4*)v_ring, dm.B,
                                               dm.T, dm.Hkv, dm.W, row_vecs, tok0);
  }
  if (pl.nseg > 0) {
    const dim3 grid(pl.nseg, dm.Hkv, dm.B);
    ProfScope ps("export_state_partial_kernel", st);
#define RATTN_EXPORT(IO, DD)                                                                                        \
  export_state_partial_kernel<IO, DD><<<grid, 256, 0, st>>>((const IO*)k, (const IO*)v, partial, dm.T, dm.Hkv, pl.Tp, \
                                                            pl.seg_len, dm.phi)
    if (dtype == 0) {
      if (dm.D == 64) RATTN_EXPORT(float, 64); else RATTN_EXPORT(float, 128);
    } else {
      if (dm.D == 64) RATTN_EXPORT(bf16_t, 64); else RATTN_EXPORT(bf16_t, 128);
    }
#undef RATTN_EXPORT
  }
  const int vecs = dm.D * dm.D / 4;
  const long long total = (long long)dm.B * dm.Hkv * vecs;
  ProfScope ps("export_state_reduce_kernel", st);
  export_state_reduce_kernel<<<(int)((total + 255) / 256), 256, 0, st>>>((const float4*)partial, (float4*)state,
                                                                         pl.nseg, vecs, total, accumulate ? 1 : 0);
}

}  // namespace rattn
