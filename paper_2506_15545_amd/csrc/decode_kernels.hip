// Decode step of the RAttention layer: one new token per sequence with constant memory
// (Sec. 2.1: cache of the last W keys;  Sec. 2.2: fixed D x D state;  Eq. 4: the linear branch reads
// the state lagging W tokens behind).  Memory bound: per (sequence, kv head) the kernel streams the
// K and V rings once (all query heads of the group share that read) and reads-modifies-writes the
// fp32 state once, with 16-byte-per-lane coalesced accesses.
#include "common.hpp"
#include "kernels.hpp"

namespace rattn {

// grid (Hkv, N), 256 threads.
template <typename IO, int D>
__global__ __launch_bounds__(256) void decode_kernel(const IO* __restrict__ q, const IO* __restrict__ k_new,
                                                     const IO* __restrict__ v_new, const int32_t* __restrict__ pos,
                                                     IO* __restrict__ k_ring, IO* __restrict__ v_ring,
                                                     float* __restrict__ state, const float* __restrict__ gs,
                                                     const float* __restrict__ gr, IO* __restrict__ o,
                                                     DecodeDims dd) {
  constexpr int HB = 4;          // query heads served per pass over the rings
  constexpr int EPL = D / 64;
  constexpr int LPR = D / 8;     // lanes per ring row (8 elements each)
  constexpr int NG = 256 / LPR;  // ring rows in flight per block
  constexpr int CG = D / 4;      // float4 column groups of the state
  constexpr int RG = 256 / CG;   // state rows in flight per block
  static_assert(RG <= NG, "partial buffer is shared");
  __shared__ float qs[HB][D];
  __shared__ float qf[HB][D];
  __shared__ float kfo[D], vo[D];
  __shared__ float xs_sh[HB][D], xr_sh[HB][D];
  __shared__ float part[NG][HB][D + 2];

  const int g = blockIdx.x, n = blockIdx.y;
  const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
  const int W = dd.W, G = dd.G, Hq = dd.Hq, Hkv = dd.Hkv;
  const int p = pos[n];
  const int slot = p % W;
  const bool evict = p >= W;
  const int nvalid = min(p + 1, W);
  IO* kr = k_ring + (size_t)(n * Hkv + g) * W * D;
  IO* vr = v_ring + (size_t)(n * Hkv + g) * W * D;
  const IO* knr = k_new + (size_t)(n * Hkv + g) * D;
  const IO* vnr = v_new + (size_t)(n * Hkv + g) * D;

  for (int hb = 0; hb < G; hb += HB) {
    const int nh = min(HB, G - hb);
    // ---- stage q, phi(q) and (first pass) phi(k_old), v_old of the token leaving the window
    for (int item = w; item < nh + (hb == 0 ? 1 : 0); item += 4) {
      float x[EPL];
      const IO* src = item < nh ? q + (size_t)(n * Hq + g * G + hb + item) * D : kr + (size_t)slot * D;
      if (item < nh || evict) {
        float m = -INFINITY;
#pragma unroll
        for (int e = 0; e < EPL; ++e) { x[e] = io_traits<IO>::ld(src + lane + 64 * e); m = fmaxf(m, x[e]); }
        m = wave_max(m);
        float ex[EPL], s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) { ex[e] = expf(x[e] - m); s += ex[e]; }
        s = 1.f / wave_sum(s);
        if (item < nh) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) { qs[item][lane + 64 * e] = x[e]; qf[item][lane + 64 * e] = ex[e] * s; }
        } else {
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            kfo[lane + 64 * e] = ex[e] * s;
            vo[lane + 64 * e] = io_traits<IO>::ld(vr + (size_t)slot * D + lane + 64 * e);
          }
        }
      }
    }
    __syncthreads();
    // ---- the new token takes the slot of the evicted one (its old content now sits in LDS)
    if (hb == 0 && tid < D) {
      kr[(size_t)slot * D + tid] = knr[tid];
      vr[(size_t)slot * D + tid] = vnr[tid];
    }
    // ---- linear branch: state += phi(k_old)^T v_old, x_r = phi(q) state
    {
      const int cg = tid % CG, rg = tid / CG;
      float xp[HB][4];
#pragma unroll
      for (int hh = 0; hh < HB; ++hh)
#pragma unroll
        for (int i = 0; i < 4; ++i) xp[hh][i] = 0.f;
      float4* Sp = reinterpret_cast<float4*>(state + (size_t)(n * Hkv + g) * D * D);
      const bool upd = evict && hb == 0;
      float4 vold = make_float4(0.f, 0.f, 0.f, 0.f);
      if (upd) vold = make_float4(vo[4 * cg], vo[4 * cg + 1], vo[4 * cg + 2], vo[4 * cg + 3]);
#pragma unroll 4
      for (int f = rg; f < D; f += RG) {
        float4 s = Sp[(size_t)f * CG + cg];
        if (upd) {
          const float kf = kfo[f];
          s.x += kf * vold.x; s.y += kf * vold.y; s.z += kf * vold.z; s.w += kf * vold.w;
          Sp[(size_t)f * CG + cg] = s;
        }
#pragma unroll
        for (int hh = 0; hh < HB; ++hh) {
          if (hh < nh) {
            const float qv = qf[hh][f];
            xp[hh][0] += qv * s.x; xp[hh][1] += qv * s.y; xp[hh][2] += qv * s.z; xp[hh][3] += qv * s.w;
          }
        }
      }
      float* red = &part[0][0][0];  // [RG][HB][D]
#pragma unroll
      for (int hh = 0; hh < HB; ++hh)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[(rg * HB + hh) * D + 4 * cg + i] = xp[hh][i];
      __syncthreads();
      for (int i = tid; i < HB * D; i += 256) {
        float s = 0.f;
        for (int r = 0; r < RG; ++r) s += red[r * HB * D + i];
        xr_sh[i / D][i % D] = s;
      }
      __syncthreads();
    }
    // ---- softmax branch over the min(p+1, W) valid slots; every row group keeps its own
    //      online-softmax partial, merged once at the end
    {
      const int grp = tid / LPR, li = tid % LPR, d0 = li * 8;
      float m[HB], l[HB], acc[HB][8], qreg[HB][8];
#pragma unroll
      for (int hh = 0; hh < HB; ++hh) {
        m[hh] = -INFINITY; l[hh] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) { acc[hh][i] = 0.f; qreg[hh][i] = hh < nh ? qs[hh][d0 + i] * dd.scale : 0.f; }
      }
      for (int i = grp; i < nvalid; i += NG) {
        const IO* kp = (i == slot) ? knr : kr + (size_t)i * D;
        const IO* vp = (i == slot) ? vnr : vr + (size_t)i * D;
        float kk[8], vv[8];
        io_traits<IO>::ld8(kp + d0, kk);
        io_traits<IO>::ld8(vp + d0, vv);
#pragma unroll
        for (int hh = 0; hh < HB; ++hh) {
          if (hh < nh) {
            float a = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) a += qreg[hh][e] * kk[e];
#pragma unroll
            for (int off = LPR / 2; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
            const float m_new = fmaxf(m[hh], a);
            const float alpha = expf(m[hh] - m_new);
            const float pe = expf(a - m_new);
            l[hh] = l[hh] * alpha + pe;
            m[hh] = m_new;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] = acc[hh][e] * alpha + pe * vv[e];
          }
        }
      }
#pragma unroll
      for (int hh = 0; hh < HB; ++hh) {
#pragma unroll
        for (int e = 0; e < 8; ++e) part[grp][hh][d0 + e] = acc[hh][e];
        if (li == 0) { part[grp][hh][D] = m[hh]; part[grp][hh][D + 1] = l[hh]; }
      }
      __syncthreads();
      for (int i = tid; i < nh * D; i += 256) {
        const int hh = i / D, d = i % D;
        float M = -INFINITY;
        for (int r = 0; r < NG; ++r) M = fmaxf(M, part[r][hh][D]);
        float num = 0.f, den = 0.f;
        for (int r = 0; r < NG; ++r) {
          const float sc = expf(part[r][hh][D] - M);
          num += sc * part[r][hh][d];
          den += sc * part[r][hh][D + 1];
        }
        xs_sh[hh][d] = num / den;
      }
      __syncthreads();
    }
    // ---- combination (Sec. 3.2)
    for (int hh = w; hh < nh; hh += 4) {
      const int h = g * G + hb + hh;
      float a[EPL], c[EPL], s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        a[e] = xs_sh[hh][lane + 64 * e]; c[e] = xr_sh[hh][lane + 64 * e];
        s1 += a[e] * a[e]; s2 += c[e] * c[e];
      }
      const float r1 = rsqrtf(wave_sum(s1) / D + dd.eps), r2 = rsqrtf(wave_sum(s2) / D + dd.eps);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int d = lane + 64 * e;
        const float g1 = gs ? gs[h * D + d] : 1.f, g2 = gr ? gr[h * D + d] : 1.f;
        io_traits<IO>::st(o + (size_t)(n * Hq + h) * D + d, g1 * a[e] * r1 + g2 * c[e] * r2);
      }
    }
    __syncthreads();
  }
}

void decode_step(const DecodeDims& dd, int dtype, const void* q, const void* k_new, const void* v_new,
                 const int32_t* pos, void* k_ring, void* v_ring, float* state, const float* gs, const float* gr,
                 void* o, hipStream_t st) {
  dim3 grid(dd.Hkv, dd.N);
  ProfScope ps("decode_kernel", st);
#define RATTN_DECODE(IO, DD)                                                                                   \
  decode_kernel<IO, DD><<<grid, 256, 0, st>>>((const IO*)q, (const IO*)k_new, (const IO*)v_new, pos, (IO*)k_ring, \
                                              (IO*)v_ring, state, gs, gr, (IO*)o, dd)
  if (dtype == 0) {
    if (dd.D == 64) RATTN_DECODE(float, 64); else RATTN_DECODE(float, 128);
  } else {
    if (dd.D == 64) RATTN_DECODE(bf16_t, 64); else RATTN_DECODE(bf16_t, 128);
  }
#undef RATTN_DECODE
}

}  // namespace rattn
