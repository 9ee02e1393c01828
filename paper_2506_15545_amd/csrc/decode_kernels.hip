// Decode step of the RAttention layer: one new token per sequence with constant memory
// (Sec. 2.1: cache of the last W keys;  Sec. 2.2: fixed D x D state;  Eq. 4: the linear branch reads
// the state lagging W tokens behind).  Memory bound: per (sequence, kv head) the kernel streams the
// K and V rings once (all query heads of the group share that read) and reads-modifies-writes the
// fp32 state once, with 16-byte-per-lane coalesced accesses.
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"

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
#pragma unroll
        for (int e = 0; e < EPL; ++e) x[e] = io_traits<IO>::ld(src + lane + 64 * e);
        float ex[EPL];
        feature_row<EPL>(x, ex, dd.phi);
        if (item < nh) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) { qs[item][lane + 64 * e] = x[e]; qf[item][lane + 64 * e] = ex[e]; }
        } else {
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            kfo[lane + 64 * e] = ex[e];
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

// Eight consecutive elements as loaded (16 or 32 bytes), converted only when consumed so that a batch of
// loads can stay in flight across the arithmetic on the previous batch.
template <typename IO> struct raw8;
template <> struct raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p);
    b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
};
template <> struct raw8<bf16_t> {
  uint4 r;
  __device__ __forceinline__ void load(const bf16_t* p) { r = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

// Two-pass variant for short rings (G <= 4 and G*W*4 bytes of scores fit beside the other LDS arrays):
// pass 1 streams K and leaves the scaled logits in LDS, the softmax runs on LDS, pass 2 streams V.  With no
// running-maximum dependency between rows, each pass keeps UNR independent 16-byte loads per lane in
// flight, which is what a bandwidth-bound kernel needs.  grid (Hkv, N), 256 threads, G*W floats of
// dynamic LDS.
//
// MFMA = true (bf16, D = 128) moves both contractions of the window branch onto the matrix cores, because
// at four query heads per ring row the fp32 vector pipe would otherwise be as busy as the memory system:
//   pass 1  S^T[key][head] = K Q^T with v_mfma_f32_16x16x32_bf16.  A is read straight from the ring in operand
//           layout (lane = key row l%16, contraction slots 8*(l/16).. of each 32-wide slice of d, i.e. 16
//           rows x 64 contiguous bytes per load instruction); B holds q (column = head, columns >= G unused).
//   pass 2  O^T[d][head] = V^T P^T.  V rows are loaded coalesced (lane = 16-byte chunk l%16 of eight rows
//           8*(l/16)+u); the k-th register pair of two rows is interleaved with one v_perm_b32 per dword,
//           which yields, for each of the 8 elements e of the chunk, an A operand whose row l%16 is the
//           output feature d = 8*(l%16)+e and whose contraction slots are the lane group's eight keys; B is
//           the matching run of eight probabilities of head l%16 (bf16, from LDS).
template <typename IO, int D, bool MFMA>
__global__ __launch_bounds__(256, 4) void decode_kernel_2pass(const IO* __restrict__ q, const IO* __restrict__ k_new,
                                                           const IO* __restrict__ v_new, const int32_t* __restrict__ pos,
                                                           IO* __restrict__ k_ring, IO* __restrict__ v_ring,
                                                           float* __restrict__ state, const float* __restrict__ gs,
                                                           const float* __restrict__ gr, IO* __restrict__ o,
                                                           DecodeDims dd) {
  constexpr int HB = 4;
  constexpr int EPL = D / 64;
  constexpr int LPR = D / 8;
  constexpr int NG = 256 / LPR;
  constexpr int CG = D / 4;
  constexpr int RG = 256 / CG;
  constexpr int UNR = 4;
  extern __shared__ float sc[];  // [G][W] logits, then unnormalised probabilities
  __shared__ float qs[HB][D];
  __shared__ float qf[HB][D];
  __shared__ float kfo[D], vo[D];
  __shared__ float xs_sh[HB][D], xr_sh[HB][D];
  __shared__ float part[4][HB][D];  // one partial per wave
  __shared__ float inv_sum[HB];

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

  // ---- stage q, phi(q), phi(k_old), v_old
  for (int item = w; item < G + 1; item += 4) {
    float x[EPL];
    const IO* src = item < G ? q + (size_t)(n * Hq + g * G + item) * D : kr + (size_t)slot * D;
    if (item < G || evict) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) x[e] = io_traits<IO>::ld(src + lane + 64 * e);
      float ex[EPL];
      feature_row<EPL>(x, ex, dd.phi);
      if (item < G) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) { qs[item][lane + 64 * e] = x[e]; qf[item][lane + 64 * e] = ex[e]; }
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          kfo[lane + 64 * e] = ex[e];
          vo[lane + 64 * e] = io_traits<IO>::ld(vr + (size_t)slot * D + lane + 64 * e);
        }
      }
    }
  }
  __syncthreads();
  if (tid < D) {
    kr[(size_t)slot * D + tid] = knr[tid];
    vr[(size_t)slot * D + tid] = vnr[tid];
  }
  // ---- linear branch: state += phi(k_old)^T v_old, x_r = phi(q) state
  auto linear_branch = [&]() {
    const int cg = tid % CG, rg = tid / CG;
    float xp[HB][4];
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
#pragma unroll
      for (int i = 0; i < 4; ++i) xp[hh][i] = 0.f;
    float4* Sp = reinterpret_cast<float4*>(state + (size_t)(n * Hkv + g) * D * D);
    float4 vold = make_float4(0.f, 0.f, 0.f, 0.f);
    if (evict) vold = make_float4(vo[4 * cg], vo[4 * cg + 1], vo[4 * cg + 2], vo[4 * cg + 3]);
    constexpr int NR = D / RG;  // rows per thread
    float4 sv[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) sv[j] = Sp[(size_t)(rg + RG * j) * CG + cg];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
      const int f = rg + RG * j;
      float4 s = sv[j];
      if (evict) {
        const float kf = kfo[f];
        s.x += kf * vold.x; s.y += kf * vold.y; s.z += kf * vold.z; s.w += kf * vold.w;
        Sp[(size_t)f * CG + cg] = s;
      }
#pragma unroll
      for (int hh = 0; hh < HB; ++hh) {
        if (hh < G) {
          const float qv = qf[hh][f];
          xp[hh][0] += qv * s.x; xp[hh][1] += qv * s.y; xp[hh][2] += qv * s.z; xp[hh][3] += qv * s.w;
        }
      }
    }
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float x = xp[hh][i];
#pragma unroll
        for (int off = CG; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
        if (lane < CG) part[w][hh][4 * cg + i] = x;
      }
    __syncthreads();
    for (int i = tid; i < HB * D; i += 256) {
      const int hh = i / D, d = i % D;
      xr_sh[hh][d] = (part[0][hh][d] + part[1][hh][d]) + (part[2][hh][d] + part[3][hh][d]);
    }
    __syncthreads();
  };
  auto window_branch = [&]() {
  if constexpr (MFMA) {
    static_assert(!MFMA || (D == 128 && sizeof(IO) == 2), "matrix-core path: bf16, D = 128");
    const int Wp = (W + 127) & ~127;
    uint16_t* pb = reinterpret_cast<uint16_t*>(sc + G * Wp);  // bf16 probabilities [G][Wp]
    const int r16 = lane & 15, q4 = lane >> 4;
    const int hcol = min(r16, G - 1);  // columns >= G of the products are never read back
    const int nset = (nvalid + 127) >> 7;  // 128 keys per workgroup step, 32 per wave
    const int rot = (int)((blockIdx.y * gridDim.x + blockIdx.x) % (unsigned)nset);
    const uint16_t* krp = reinterpret_cast<const uint16_t*>(kr);
    const uint16_t* vrp = reinterpret_cast<const uint16_t*>(vr);
    const uint16_t* knp = reinterpret_cast<const uint16_t*>(knr);
    const uint16_t* vnp = reinterpret_cast<const uint16_t*>(vnr);
    // ---- pass 1
    {
      bf16x8_t qb[4];
      const uint16_t* qp = reinterpret_cast<const uint16_t*>(q) + (size_t)(n * Hq + g * G + hcol) * D;
#pragma unroll
      for (int j = 0; j < 4; ++j) qb[j] = *reinterpret_cast<const bf16x8_t*>(qp + 32 * j + 8 * q4);
      auto fetch = [&](bf16x8_t (&dst)[8], int set) {
        const int base = (set * 4 + w) * 32;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const int r = base + 16 * c + r16;
          const int rc = r < nvalid ? r : 0;
          const uint16_t* rp = rc == slot ? knp : krp + (size_t)rc * D;
#pragma unroll
          for (int j = 0; j < 4; ++j) dst[c * 4 + j] = *reinterpret_cast<const bf16x8_t*>(rp + 32 * j + 8 * q4);
        }
      };
      bf16x8_t cur[8], nxt[8];
      fetch(cur, rot);
      for (int it = 0; it < nset; ++it) {
        const int set = it + rot < nset ? it + rot : it + rot - nset;
        const bool more = it + 1 < nset;
        if (more) fetch(nxt, set + 1 < nset ? set + 1 : 0);
        const int base = (set * 4 + w) * 32;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          f32x4_t a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int j = 0; j < 4; ++j) a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur[c * 4 + j], qb[j], a, 0, 0, 0);
          // lane (head r16, group q4): a[i] = logit of key base + 16c + 4*q4 + i
          if (r16 < G) {
            a *= dd.scale;
            *reinterpret_cast<f32x4_t*>(sc + r16 * Wp + base + 16 * c + 4 * q4) = a;
          }
        }
        if (more) {
#pragma unroll
          for (int u = 0; u < 8; ++u) cur[u] = nxt[u];
        }
      }
    }
    __syncthreads();
    // ---- softmax, one wave per head; slots past nvalid get probability 0
    for (int hh = w; hh < G; hh += 4) {
      float m = -INFINITY;
      for (int r = lane; r < nvalid; r += 64) m = fmaxf(m, sc[hh * Wp + r]);
      m = wave_max(m);
      float sum = 0.f;
      for (int r = lane; r < nset * 128; r += 64) {
        const float e = r < nvalid ? expf(sc[hh * Wp + r] - m) : 0.f;
        pb[hh * Wp + r] = f32_to_bf16(e);
        sum += e;
      }
      sum = wave_sum(sum);
      if (lane == 0) inv_sum[hh] = 1.f / sum;
    }
    __syncthreads();
    // ---- pass 2
    {
      typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
      auto fetch = [&](u32x4_t (&dst)[8], int set) {
        const int base = (set * 4 + w) * 32 + 8 * q4;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int r = base + u;
          const int rc = r < nvalid ? r : 0;
          const uint16_t* rp = rc == slot ? vnp : vrp + (size_t)rc * D;
          dst[u] = *reinterpret_cast<const u32x4_t*>(rp + 8 * r16);
        }
      };
      f32x4_t acc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      u32x4_t cur[8], nxt[8];
      fetch(cur, rot);
      for (int it = 0; it < nset; ++it) {
        const int set = it + rot < nset ? it + rot : it + rot - nset;
        const bool more = it + 1 < nset;
        if (more) fetch(nxt, set + 1 < nset ? set + 1 : 0);
        const int base = (set * 4 + w) * 32 + 8 * q4;
        const bf16x8_t pv = *reinterpret_cast<const bf16x8_t*>(pb + hcol * Wp + base);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int j = e >> 1;
          const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
          u32x4_t a;
          a[0] = __builtin_amdgcn_perm(cur[1][j], cur[0][j], sel);
          a[1] = __builtin_amdgcn_perm(cur[3][j], cur[2][j], sel);
          a[2] = __builtin_amdgcn_perm(cur[5][j], cur[4][j], sel);
          a[3] = __builtin_amdgcn_perm(cur[7][j], cur[6][j], sel);
          acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), pv, acc[e], 0, 0, 0);
        }
        if (more) {
#pragma unroll
          for (int u = 0; u < 8; ++u) cur[u] = nxt[u];
        }
      }
      // lane (head r16, group q4): acc[e][i] = x_s partial of feature d = 8*(4*q4 + i) + e
      if (r16 < G) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
          for (int i = 0; i < 4; ++i) part[w][r16][8 * (4 * q4 + i) + e] = acc[e][i];
      }
      __syncthreads();
      for (int i = tid; i < G * D; i += 256) {
        const int hh = i / D, d = i % D;
        xs_sh[hh][d] = ((part[0][hh][d] + part[1][hh][d]) + (part[2][hh][d] + part[3][hh][d])) * inv_sum[hh];
      }
      __syncthreads();
    }
  } else {
  const int grp = tid / LPR, li = tid % LPR, d0 = li * 8;
  // Workgroups run in lockstep over rings that lie a multiple of W*D elements apart; starting each one at a
  // different batch of rows spreads the simultaneous requests over the memory channels.
  const int nbatch = (nvalid + NG * UNR - 1) / (NG * UNR);
  const int rot = (int)((blockIdx.y * gridDim.x + blockIdx.x) % (unsigned)nbatch);
  // ---- pass 1: logits of all valid slots
  {
    float qreg[HB][8];
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
#pragma unroll
      for (int i = 0; i < 8; ++i) qreg[hh][i] = hh < G ? qs[hh][d0 + i] * dd.scale : 0.f;
    auto fetch = [&](raw8<IO> (&dst)[UNR], int base) {
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int r = base + u * NG + grp;
        const int rc = r < nvalid ? r : 0;
        dst[u].load((rc == slot ? knr : kr + (size_t)rc * D) + d0);
      }
    };
    raw8<IO> cur[UNR], nxt[UNR];
    fetch(cur, rot * (NG * UNR));
    for (int it = 0; it < nbatch; ++it) {
      const int bi = it + rot < nbatch ? it + rot : it + rot - nbatch;
      const int base = bi * (NG * UNR);
      const bool more = it + 1 < nbatch;
      if (more) fetch(nxt, (bi + 1 < nbatch ? bi + 1 : 0) * (NG * UNR));
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int r = base + u * NG + grp;
        float kk[8];
        cur[u].unpack(kk);
#pragma unroll
        for (int hh = 0; hh < HB; ++hh) {
          if (hh < G) {
            float a = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) a += qreg[hh][e] * kk[e];
#pragma unroll
            for (int off = LPR / 2; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
            if (li == 0 && r < nvalid) sc[hh * W + r] = a;
          }
        }
      }
      if (more) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) cur[u] = nxt[u];
      }
    }
  }
  __syncthreads();
  // ---- softmax over the logits, one wave per head
  for (int hh = w; hh < G; hh += 4) {
    float m = -INFINITY;
    for (int r = lane; r < nvalid; r += 64) m = fmaxf(m, sc[hh * W + r]);
    m = wave_max(m);
    float s = 0.f;
    for (int r = lane; r < nvalid; r += 64) {
      const float e = expf(sc[hh * W + r] - m);
      sc[hh * W + r] = e;
      s += e;
    }
    s = wave_sum(s);
    if (lane == 0) inv_sum[hh] = 1.f / s;
  }
  __syncthreads();
  // ---- pass 2: x_s = P V
  {
    float acc[HB][8];
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[hh][i] = 0.f;
    auto fetch = [&](raw8<IO> (&dst)[UNR], int base) {
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int r = base + u * NG + grp;
        const int rc = r < nvalid ? r : 0;
        dst[u].load((rc == slot ? vnr : vr + (size_t)rc * D) + d0);
      }
    };
    raw8<IO> cur[UNR], nxt[UNR];
    fetch(cur, rot * (NG * UNR));
    for (int it = 0; it < nbatch; ++it) {
      const int bi = it + rot < nbatch ? it + rot : it + rot - nbatch;
      const int base = bi * (NG * UNR);
      const bool more = it + 1 < nbatch;
      if (more) fetch(nxt, (bi + 1 < nbatch ? bi + 1 : 0) * (NG * UNR));
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int r = base + u * NG + grp;
        if (r < nvalid) {
          float vv[8];
          cur[u].unpack(vv);
#pragma unroll
          for (int hh = 0; hh < HB; ++hh) {
            if (hh < G) {
              const float pe = sc[hh * W + r];
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[hh][e] += pe * vv[e];
            }
          }
        }
      }
      if (more) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) cur[u] = nxt[u];
      }
    }
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = acc[hh][e];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
        if (lane < LPR) part[w][hh][d0 + e] = x;
      }
    __syncthreads();
    for (int i = tid; i < G * D; i += 256) {
      const int hh = i / D, d = i % D;
      xs_sh[hh][d] = ((part[0][hh][d] + part[1][hh][d]) + (part[2][hh][d] + part[3][hh][d])) * inv_sum[hh];
    }
    __syncthreads();
  }
  }
  };
  // Co-resident workgroups start in lockstep; running the two branches in opposite order in half of them
  // lets one group stream while the other sits in a reduction or softmax bubble.
  if (((blockIdx.y >> 5) ^ blockIdx.y) & 1) {
    linear_branch();
    window_branch();
  } else {
    window_branch();
    linear_branch();
  }
  // ---- combination (Sec. 3.2)
  for (int hh = w; hh < G; hh += 4) {
    const int h = g * G + hh;
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
}

void decode_step(const DecodeDims& dd, int dtype, const void* q, const void* k_new, const void* v_new,
                 const int32_t* pos, void* k_ring, void* v_ring, float* state, const float* gs, const float* gr,
                 void* o, hipStream_t st) {
  dim3 grid(dd.Hkv, dd.N);
  ProfScope ps("decode_kernel", st);
  const size_t score_bytes = (size_t)dd.G * dd.W * sizeof(float);
  const size_t mfma_bytes = (size_t)dd.G * ((dd.W + 127) & ~127) * 6;  // fp32 logits + bf16 probabilities
#define RATTN_DECODE2(IO, DD, MF, BYTES)                                                                        \
  decode_kernel_2pass<IO, DD, MF><<<grid, 256, BYTES, st>>>((const IO*)q, (const IO*)k_new, (const IO*)v_new, pos, \
                                                            (IO*)k_ring, (IO*)v_ring, state, gs, gr, (IO*)o, dd)
  if (dtype == 1 && dd.D == 128 && dd.G <= 4 && mfma_bytes <= 24576) {
    RATTN_DECODE2(bf16_t, 128, true, mfma_bytes);
    return;
  }
  if (dd.G <= 4 && score_bytes <= 16384) {
    if (dtype == 0) {
      if (dd.D == 64) RATTN_DECODE2(float, 64, false, score_bytes); else RATTN_DECODE2(float, 128, false, score_bytes);
    } else {
      if (dd.D == 64) RATTN_DECODE2(bf16_t, 64, false, score_bytes); else RATTN_DECODE2(bf16_t, 128, false, score_bytes);
    }
    return;
  }
#undef RATTN_DECODE2
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
