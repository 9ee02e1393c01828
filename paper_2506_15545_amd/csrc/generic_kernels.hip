// General-shape kernels of librattn: any T, any window W >= 1, D in {64,128}, fp32 or bf16 I/O,
// fp32 arithmetic on the vector ALUs.  One wavefront owns one query (or one key) row; the other
// operand's rows are spread over the 64 lanes.  These kernels serve fp32 tensors and every shape
// the MFMA kernels do not cover; they follow the same decomposition:
//   softmax branch  : Sec. 2.1 (windowed softmax, online normalisation)
//   linear branch   : Eqs. 2-4 (chunk states S_[j], inter-chunk product + intra-chunk masked product,
//                     read at lag W), phi (row softmax, or the ablation's ReLU / identity of Sec. 4.5)
//                     computed in-kernel, never stored
//   combination     : Sec. 3.2 (two RMS norms with per-head gains)
// Element d of a row lives in lane d % 64, register d / 64.
#include "common.hpp"
#include "kernels.hpp"

namespace rattn {

template <typename IO, int D> struct Row {
  static constexpr int EPL = D / 64;
  float x[EPL];
  __device__ __forceinline__ void load(const IO* p) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) x[e] = io_traits<IO>::ld(p + lane_id() + 64 * e);
  }
  __device__ __forceinline__ void store(IO* p) const {
#pragma unroll
    for (int e = 0; e < EPL; ++e) io_traits<IO>::st(p + lane_id() + 64 * e, x[e]);
  }
  __device__ __forceinline__ float get(int d) const { return bcast(x[d / 64], d % 64); }  // d compile-time after unrolling
  __device__ __forceinline__ float sumsq() const {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) s += x[e] * x[e];
    return wave_sum(s);
  }
  __device__ __forceinline__ float dot(const Row& o) const {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) s += x[e] * o.x[e];
    return wave_sum(s);
  }
  // in place feature map over the D features
  __device__ __forceinline__ void feature(int phi) { feature_row<EPL>(x, x, phi); }
};

// <row held across the wave, row read privately by this lane>
template <typename RT, int D, typename IO2>
__device__ __forceinline__ float lane_dot(const Row<RT, D>& r, const IO2* own) {
  float a = 0.f;
#pragma unroll
  for (int c = 0; c < D / 8; ++c) {
    float t[8];
    io_traits<IO2>::ld8(own + c * 8, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) a += r.get(c * 8 + i) * t[i];
  }
  return a;
}

// row statistics (m, z) of the row this lane reads privately: max and sum(exp(x - max)) for softmax, (0, 1) otherwise
template <int D, typename IO>
__device__ __forceinline__ void lane_feature_stats(const IO* own, float& m, float& z, int phi) {
  if (phi != PHI_SOFTMAX) { m = 0.f; z = 1.f; return; }
  m = -INFINITY;
#pragma unroll
  for (int c = 0; c < D / 8; ++c) {
    float t[8];
    io_traits<IO>::ld8(own + c * 8, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, t[i]);
  }
  z = 0.f;
#pragma unroll
  for (int c = 0; c < D / 8; ++c) {
    float t[8];
    io_traits<IO>::ld8(own + c * 8, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) z += expf(t[i] - m);
  }
}

// sum_f r[f] * feat(own[f], m)   (r spread over the wave, own row private)
template <typename RT, int D, typename IO>
__device__ __forceinline__ float lane_dot_feat(const Row<RT, D>& r, const IO* own, float m, int phi) {
  float a = 0.f;
#pragma unroll
  for (int c = 0; c < D / 8; ++c) {
    float t[8];
    io_traits<IO>::ld8(own + c * 8, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) a += r.get(c * 8 + i) * feat(t[i], m, phi);
  }
  return a;
}

// ------------------------------------------------------------------------------------------------
// Chunk-boundary states of the linear branch (Eq. 2): exclusive prefix (REV=false) or suffix
// (REV=true) sums over chunks of  sum_t phi(a_t)^T b_t,  t' in [0,Tp), token index t' + off,
// summed over the GA heads g*GA .. g*GA+GA-1 of a tensor with H heads.
// out[(b*Hkv+g)*nst + j] is the D x D state seen by chunk j.  grid (D/16, Hkv, B), 256 threads:
// the block owns a 16-column slice of the state and walks the tokens in order.
template <typename AT, typename BT, int D, bool REV>
__global__ __launch_bounds__(256) void gen_scan_kernel(const AT* __restrict__ a, const BT* __restrict__ bsrc,
                                                       float* __restrict__ out, int T, int H, int GA, int off,
                                                       int Tp, int C, int nst, int phi) {
  constexpr int TB = 16;
  constexpr int CPT = D / 16;    // state columns per thread
  constexpr int TPR = 16 / CPT;  // threads per state row
  __shared__ float af[TB][D];
  __shared__ float bs[TB][16];
  const int slice = blockIdx.x, g = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int tid = threadIdx.x, f = tid / TPR, c0 = (tid % TPR) * CPT;
  const int w = wave_id();
  float S[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) S[c] = 0.f;
  float* obase = out + (size_t)(b * Hkv + g) * nst * D * D;
  for (int jj = 0; jj < nst; ++jj) {
    const int j = REV ? nst - 1 - jj : jj;
    float* dst = obase + (size_t)j * D * D + (size_t)f * D + slice * 16 + c0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) dst[c] = S[c];
    if (jj == nst - 1) break;
    const int lo = j * C, hi = min(lo + C, Tp);
    for (int ga = 0; ga < GA; ++ga) {
      const int head = g * GA + ga;
      for (int t0 = lo; t0 < hi; t0 += TB) {
        const int n = min(TB, hi - t0);
        __syncthreads();
        for (int tt = w; tt < n; tt += 4) {
          Row<AT, D> r;
          r.load(a + ((size_t)(b * T + t0 + tt + off) * H + head) * D);
          r.feature(phi);
#pragma unroll
          for (int e = 0; e < D / 64; ++e) af[tt][lane_id() + 64 * e] = r.x[e];
        }
        if (tid < n * 16) {
          const int tt = tid / 16, c = tid % 16;
          bs[tt][c] = io_traits<BT>::ld(bsrc + ((size_t)(b * T + t0 + tt + off) * H + head) * D + slice * 16 + c);
        }
        __syncthreads();
        for (int tt = 0; tt < n; ++tt) {
          const float av = af[tt][f];
#pragma unroll
          for (int c = 0; c < CPT; ++c) S[c] += av * bs[tt][c0 + c];
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Forward: one wave per query row, QPW rows per wave.  grid (ceil(T/(4*QPW)), Hq, B), 256 threads.
constexpr int GEN_QPW = 4;

template <typename IO, typename ST, int D>
__global__ __launch_bounds__(256) void gen_fwd_kernel(const IO* __restrict__ q, const IO* __restrict__ k,
                                                      const IO* __restrict__ v, const float* __restrict__ gs,
                                                      const float* __restrict__ gr,
                                                      const float* __restrict__ states, IO* __restrict__ o,
                                                      ST* __restrict__ xs_out, ST* __restrict__ xr_out,
                                                      float* __restrict__ lse_out, float* __restrict__ rs_out,
                                                      float* __restrict__ rr_out, LayerDims dm) {
  constexpr int EPL = D / 64;
  const int h = blockIdx.y, b = blockIdx.z, g = h / dm.G;
  const int lane = lane_id();
  const int T = dm.T, W = dm.W, C = dm.C, Hq = dm.Hq, Hkv = dm.Hkv;
  for (int qi = 0; qi < GEN_QPW; ++qi) {
    const int t = (blockIdx.x * 4 + wave_id()) * GEN_QPW + qi;
    if (t >= T) break;
    const size_t qoff = ((size_t)(b * T + t) * Hq + h) * D;
    Row<IO, D> qv;
    qv.load(q + qoff);
    // ---- softmax branch over keys max(0,t-W+1)..t
    float m = -INFINITY, l = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    const int s_lo = max(0, t - W + 1);
    for (int base = s_lo; base <= t; base += 64) {
      const int s = base + lane;
      const bool valid = s <= t;
      const int sc = valid ? s : t;
      float a = dm.scale * lane_dot(qv, k + ((size_t)(b * T + sc) * Hkv + g) * D);
      a = valid ? a : -INFINITY;
      const float m_new = fmaxf(m, wave_max(a));
      const float alpha = expf(m - m_new);
      const float p = valid ? expf(a - m_new) : 0.f;
      l = l * alpha + wave_sum(p);
      m = m_new;
      const int n = min(64, t - base + 1);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
      for (int j = 0; j < n; ++j) {
        const float pj = bcast(p, j);
        const IO* vr = v + ((size_t)(b * T + base + j) * Hkv + g) * D;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += pj * io_traits<IO>::ld(vr + lane + 64 * e);
      }
    }
    Row<float, D> xs;
    const float inv_l = 1.f / l;
#pragma unroll
    for (int e = 0; e < EPL; ++e) xs.x[e] = acc[e] * inv_l;
    // ---- linear branch: phi(q) S_[j] + intra-chunk part over keys jC..t-W
    Row<float, D> xr;
#pragma unroll
    for (int e = 0; e < EPL; ++e) xr.x[e] = 0.f;
    const int pidx = t - W;
    if (pidx >= 0) {
      Row<IO, D> qf = qv;
      qf.feature(dm.phi);
      const int j = pidx / C;
      const float* S = states + ((size_t)(b * Hkv + g) * dm.nst + j) * D * D;
#pragma unroll 8
      for (int f = 0; f < D; ++f) {
        const float qff = bcast(qf.x[f / 64], f % 64);
#pragma unroll
        for (int e = 0; e < EPL; ++e) xr.x[e] += qff * S[(size_t)f * D + lane + 64 * e];
      }
      for (int base = j * C; base <= pidx; base += 64) {
        const int s = base + lane;
        const bool valid = s <= pidx;
        const int sc = valid ? s : pidx;
        const IO* kr = k + ((size_t)(b * T + sc) * Hkv + g) * D;
        float mk, zk;
        lane_feature_stats<D>(kr, mk, zk, dm.phi);
        float c = lane_dot_feat(qf, kr, mk, dm.phi) / zk;
        c = valid ? c : 0.f;
        const int n = min(64, pidx - base + 1);
        for (int jj = 0; jj < n; ++jj) {
          const float cj = bcast(c, jj);
          const IO* vr = v + ((size_t)(b * T + base + jj) * Hkv + g) * D;
#pragma unroll
          for (int e = 0; e < EPL; ++e) xr.x[e] += cj * io_traits<IO>::ld(vr + lane + 64 * e);
        }
      }
    }
    // ---- combination
    const float r_s = rsqrtf(xs.sumsq() / D + dm.eps);
    const float r_r = rsqrtf(xr.sumsq() / D + dm.eps);
    Row<float, D> out;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int d = lane + 64 * e;
      const float g1 = gs ? gs[h * D + d] : 1.f, g2 = gr ? gr[h * D + d] : 1.f;
      out.x[e] = g1 * xs.x[e] * r_s + g2 * xr.x[e] * r_r;
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) io_traits<IO>::st(o + qoff + lane + 64 * e, out.x[e]);
    if (xs_out) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        io_traits<ST>::st(xs_out + qoff + lane + 64 * e, xs.x[e]);
        io_traits<ST>::st(xr_out + qoff + lane + 64 * e, xr.x[e]);
      }
      if (lane == 0) {
        const size_t so = (size_t)(b * Hq + h) * T + t;
        lse_out[so] = m + logf(l);
        rs_out[so] = r_s;
        rr_out[so] = r_r;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Backward, step 1: through the two RMS norms (Sec. 3.2).  For y = g*x*r, r = (mean x^2+eps)^-1/2:
//   dx = r*(g*dy) - x*r^3*mean(g*dy*x),   dgamma += dy*x*r,   delta = <dx_s, x_s>.
// grid (RB, Hq): block rb walks rows rb, rb+RB, ... of the B*T rows of head h; each wave keeps
// per-feature dgamma partials, combined across the 4 waves at the end -> dgpart[2][RB][Hq][D].
template <typename IO, typename ST, int D>
__global__ __launch_bounds__(256) void gen_bwd_prep_kernel(const IO* __restrict__ dO, const ST* __restrict__ xs_in,
                                                           const ST* __restrict__ xr_in,
                                                           const float* __restrict__ rs_in,
                                                           const float* __restrict__ rr_in,
                                                           const float* __restrict__ gs, const float* __restrict__ gr,
                                                           float* __restrict__ dxs, float* __restrict__ dxr,
                                                           float* __restrict__ delta, float* __restrict__ dgpart,
                                                           LayerDims dm) {
  constexpr int EPL = D / 64;
  __shared__ float red[2][4][D];
  const int h = blockIdx.y, RB = gridDim.x, lane = lane_id(), w = wave_id();
  const int rows = dm.B * dm.T;
  float dg1[EPL], dg2[EPL], g1[EPL], g2[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    dg1[e] = dg2[e] = 0.f;
    g1[e] = gs ? gs[h * D + lane + 64 * e] : 1.f;
    g2[e] = gr ? gr[h * D + lane + 64 * e] : 1.f;
  }
  for (int r = blockIdx.x * 4 + w; r < rows; r += RB * 4) {
    const int b = r / dm.T, t = r % dm.T;
    const size_t off = ((size_t)r * dm.Hq + h) * D;
    const size_t so = (size_t)(b * dm.Hq + h) * dm.T + t;
    Row<IO, D> dy;
    Row<ST, D> xs, xr;
    dy.load(dO + off); xs.load(xs_in + off); xr.load(xr_in + off);
    const float r_s = rs_in[so], r_r = rr_in[so];
    float m1 = 0.f, m2 = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) { m1 += g1[e] * dy.x[e] * xs.x[e]; m2 += g2[e] * dy.x[e] * xr.x[e]; }
    m1 = wave_sum(m1) / D; m2 = wave_sum(m2) / D;
    float dl = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float a = r_s * g1[e] * dy.x[e] - xs.x[e] * r_s * r_s * r_s * m1;
      const float c = r_r * g2[e] * dy.x[e] - xr.x[e] * r_r * r_r * r_r * m2;
      dxs[off + lane + 64 * e] = a;
      dxr[off + lane + 64 * e] = c;
      dl += a * xs.x[e];
      dg1[e] += dy.x[e] * xs.x[e] * r_s;
      dg2[e] += dy.x[e] * xr.x[e] * r_r;
    }
    dl = wave_sum(dl);
    if (lane == 0) delta[so] = dl;
  }
#pragma unroll
  for (int e = 0; e < EPL; ++e) { red[0][w][lane + 64 * e] = dg1[e]; red[1][w][lane + 64 * e] = dg2[e]; }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * D; i += 256) {
    const int which = i / D, d = i % D;
    const float s = red[which][0][d] + red[which][1][d] + red[which][2][d] + red[which][3][d];
    dgpart[((size_t)(which * RB + blockIdx.x) * dm.Hq + h) * D + d] = s;
  }
}

// dgamma[h][d] = sum over the RB partials, in a fixed order.  grid (ceil(Hq*D/256)), 256 threads.
__global__ void gen_dgamma_reduce_kernel(const float* __restrict__ dgpart, float* __restrict__ dgs,
                                         float* __restrict__ dgr, int RB, int HD) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= HD) return;
  float s1 = 0.f, s2 = 0.f;
  for (int r = 0; r < RB; ++r) { s1 += dgpart[(size_t)r * HD + i]; s2 += dgpart[(size_t)(RB + r) * HD + i]; }
  if (dgs) dgs[i] = s1;
  if (dgr) dgr[i] = s2;
}

// ------------------------------------------------------------------------------------------------
// Backward, dq: one wave per query row (layout as the forward).
//   softmax branch: p = exp(scale q.k - lse), dp = <dx_s, v_s>, da = p(dp - delta), dq += scale*da*k_s
//                   (delta recomputed from p and dp, and written back, when the window fits one pass: W <= 64)
//   linear branch : dphi(q) = S_[j] dx_r + sum_{intra} <dx_r, v_s> phi(k_s);  dq += phi(q)*(dphi - <dphi,phi(q)>)
//                   (softmax map; ReLU passes dphi where q > 0, identity passes it unchanged)
template <typename IO, int D>
__global__ __launch_bounds__(256) void gen_bwd_dq_kernel(const IO* __restrict__ q, const IO* __restrict__ k,
                                                         const IO* __restrict__ v, const float* __restrict__ dxs,
                                                         const float* __restrict__ dxr, float* delta,
                                                         const float* __restrict__ lse,
                                                         const float* __restrict__ states, IO* __restrict__ dq,
                                                         LayerDims dm) {
  constexpr int EPL = D / 64;
  const int h = blockIdx.y, b = blockIdx.z, g = h / dm.G;
  const int lane = lane_id();
  const int T = dm.T, W = dm.W, C = dm.C, Hq = dm.Hq, Hkv = dm.Hkv;
  for (int qi = 0; qi < GEN_QPW; ++qi) {
    const int t = (blockIdx.x * 4 + wave_id()) * GEN_QPW + qi;
    if (t >= T) break;
    const size_t qoff = ((size_t)(b * T + t) * Hq + h) * D;
    const size_t so = (size_t)(b * Hq + h) * T + t;
    Row<IO, D> qv;
    qv.load(q + qoff);
    Row<float, D> gxs, gxr;
    gxs.load(dxs + qoff); gxr.load(dxr + qoff);
    float dl = delta[so];
    const float ls = lse[so];
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    const int s_lo = max(0, t - W + 1);
    for (int base = s_lo; base <= t; base += 64) {
      const int s = base + lane;
      const bool valid = s <= t;
      const int sc = valid ? s : t;
      const size_t ko = ((size_t)(b * T + sc) * Hkv + g) * D;
      const float a = dm.scale * lane_dot(qv, k + ko);
      const float p = valid ? expf(a - ls) : 0.f;
      const float dp = lane_dot(gxs, v + ko);
      if (W <= 64) {
        // The window fits one pass of the wave: delta = sum_j p_j dp_j from the very p and dp that form da, instead
        // of <dx_s, x_s> with the stored x_s.  For windows of a few keys p is nearly one-hot and p (dp - delta)
        // cancels; the rounding of a bf16-stored x_s would be what is left.  The dk/dv kernel reads it back.
        dl = wave_sum(p * dp);
        if (lane == 0) delta[so] = dl;
      }
      const float da = p * (dp - dl);
      const int n = min(64, t - base + 1);
      for (int j = 0; j < n; ++j) {
        const float daj = bcast(da, j);
        const IO* kr = k + ((size_t)(b * T + base + j) * Hkv + g) * D;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += daj * io_traits<IO>::ld(kr + lane + 64 * e);
      }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= dm.scale;
    const int pidx = t - W;
    if (pidx >= 0) {
      Row<IO, D> qf = qv;
      qf.feature(dm.phi);
      const int j = pidx / C;
      const float* S = states + ((size_t)(b * Hkv + g) * dm.nst + j) * D * D;
      Row<float, D> dqf;
#pragma unroll
      for (int e = 0; e < EPL; ++e) dqf.x[e] = lane_dot(gxr, S + (size_t)(lane + 64 * e) * D);
      for (int base = j * C; base <= pidx; base += 64) {
        const int s = base + lane;
        const bool valid = s <= pidx;
        const int sc = valid ? s : pidx;
        const size_t ko = ((size_t)(b * T + sc) * Hkv + g) * D;
        float mk, zk;
        lane_feature_stats<D>(k + ko, mk, zk, dm.phi);
        float coef = lane_dot(gxr, v + ko) / zk;
        coef = valid ? coef : 0.f;
        const int n = min(64, pidx - base + 1);
        for (int jj = 0; jj < n; ++jj) {
          const float cf = bcast(coef, jj), mj = bcast(mk, jj);
          const IO* kr = k + ((size_t)(b * T + base + jj) * Hkv + g) * D;
#pragma unroll
          for (int e = 0; e < EPL; ++e) dqf.x[e] += cf * feat(io_traits<IO>::ld(kr + lane + 64 * e), mj, dm.phi);
        }
      }
      float inner = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) inner += dqf.x[e] * qf.x[e];
      inner = wave_sum(inner);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] += feat_bwd(qv.x[e], qf.x[e], dqf.x[e], inner, dm.phi);
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) io_traits<IO>::st(dq + qoff + lane + 64 * e, acc[e]);
  }
}

// ------------------------------------------------------------------------------------------------
// Backward, dk and dv: one wave per key row of a KV head; the G query heads of the group are
// visited in turn, so no atomics are needed.  `rstates` are the reverse-time chunk states
// R_[j] = sum over query chunks after j of phi(q)^T dx_r (summed over the group's heads).
template <typename IO, int D>
__global__ __launch_bounds__(256) void gen_bwd_dkv_kernel(const IO* __restrict__ q, const IO* __restrict__ k,
                                                          const IO* __restrict__ v, const float* __restrict__ dxs,
                                                          const float* __restrict__ dxr,
                                                          const float* __restrict__ delta,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ rstates, IO* __restrict__ dk,
                                                          IO* __restrict__ dv, LayerDims dm) {
  constexpr int EPL = D / 64;
  const int g = blockIdx.y, b = blockIdx.z;
  const int lane = lane_id();
  const int T = dm.T, W = dm.W, C = dm.C, Hq = dm.Hq, Hkv = dm.Hkv, G = dm.G;
  const int Tp = max(T - W, 0);
  for (int ki = 0; ki < GEN_QPW; ++ki) {
    const int s = (blockIdx.x * 4 + wave_id()) * GEN_QPW + ki;
    if (s >= T) break;
    const size_t koff = ((size_t)(b * T + s) * Hkv + g) * D;
    Row<IO, D> kv, vv;
    kv.load(k + koff); vv.load(v + koff);
    Row<IO, D> kf = kv;
    kf.feature(dm.phi);
    float dka[EPL], dva[EPL];
    Row<float, D> dkf;
#pragma unroll
    for (int e = 0; e < EPL; ++e) dka[e] = dva[e] = dkf.x[e] = 0.f;
    const int tmax = min(s + W - 1, T - 1);
    const bool in_lin = s < Tp;
    const int j = s / C;
    const int tpmax = min((j + 1) * C, Tp) - 1;
    for (int hh = 0; hh < G; ++hh) {
      const int h = g * G + hh;
      const size_t sbase = (size_t)(b * Hq + h) * T;
      for (int base = s; base <= tmax; base += 64) {
        const int t = base + lane;
        const bool valid = t <= tmax;
        const int tc = valid ? t : tmax;
        const size_t qo = ((size_t)(b * T + tc) * Hq + h) * D;
        const float a = dm.scale * lane_dot(kv, q + qo);
        const float p = valid ? expf(a - lse[sbase + tc]) : 0.f;
        const float dp = lane_dot(vv, dxs + qo);
        const float da = p * (dp - delta[sbase + tc]);
        const int n = min(64, tmax - base + 1);
        for (int jj = 0; jj < n; ++jj) {
          const float pj = bcast(p, jj), daj = bcast(da, jj);
          const size_t ro = ((size_t)(b * T + base + jj) * Hq + h) * D;
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            dva[e] += pj * dxs[ro + lane + 64 * e];
            dka[e] += daj * io_traits<IO>::ld(q + ro + lane + 64 * e);
          }
        }
      }
      if (in_lin) {
        for (int base = s; base <= tpmax; base += 64) {
          const int tp = base + lane;
          const bool valid = tp <= tpmax;
          const int t = (valid ? tp : tpmax) + W;
          const size_t qo = ((size_t)(b * T + t) * Hq + h) * D;
          float mq, zq;
          lane_feature_stats<D>(q + qo, mq, zq, dm.phi);
          float c = lane_dot_feat(kf, q + qo, mq, dm.phi) / zq;
          float coef = lane_dot(vv, dxr + qo) / zq;
          c = valid ? c : 0.f;
          coef = valid ? coef : 0.f;
          const int n = min(64, tpmax - base + 1);
          for (int jj = 0; jj < n; ++jj) {
            const float cj = bcast(c, jj), cf = bcast(coef, jj), mj = bcast(mq, jj);
            const size_t ro = ((size_t)(b * T + base + jj + W) * Hq + h) * D;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
              dva[e] += cj * dxr[ro + lane + 64 * e];
              dkf.x[e] += cf * feat(io_traits<IO>::ld(q + ro + lane + 64 * e), mj, dm.phi);
            }
          }
        }
      }
    }
    if (in_lin) {
      const float* R = rstates + ((size_t)(b * Hkv + g) * dm.nst + j) * D * D;
#pragma unroll 8
      for (int f = 0; f < D; ++f) {
        const float kff = bcast(kf.x[f / 64], f % 64);
#pragma unroll
        for (int e = 0; e < EPL; ++e) dva[e] += kff * R[(size_t)f * D + lane + 64 * e];
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) dkf.x[e] += lane_dot(vv, R + (size_t)(lane + 64 * e) * D);
    }
    float inner = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) inner += dkf.x[e] * kf.x[e];
    inner = wave_sum(inner);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      io_traits<IO>::st(dk + koff + lane + 64 * e,
                        dm.scale * dka[e] + feat_bwd(kv.x[e], kf.x[e], dkf.x[e], inner, dm.phi));
      io_traits<IO>::st(dv + koff + lane + 64 * e, dva[e]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// host launchers
template <typename IO, typename ST, int D>
static void launch_fwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs,
                       const float* gr, void* o, const SavedPtrs& sv, float* states, hipStream_t st) {
  if (dm.nst > 0) {
    ProfScope ps("gen_scan_kernel", st);
    gen_scan_kernel<IO, IO, D, false><<<dim3(D / 16, dm.Hkv, dm.B), 256, 0, st>>>(
        (const IO*)k, (const IO*)v, states, dm.T, dm.Hkv, 1, 0, dm.T - dm.W, dm.C, dm.nst, dm.phi);
  }
  dim3 grid((dm.T + 4 * GEN_QPW - 1) / (4 * GEN_QPW), dm.Hq, dm.B);
  ProfScope ps("gen_fwd_kernel", st);
  gen_fwd_kernel<IO, ST, D><<<grid, 256, 0, st>>>((const IO*)q, (const IO*)k, (const IO*)v, gs, gr, states, (IO*)o,
                                                  (ST*)sv.xs, (ST*)sv.xr, sv.lse, sv.rs, sv.rr, dm);
}

template <typename IO, typename ST, int D>
static void launch_bwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs,
                       const float* gr, const SavedPtrs& sv, const void* dO, void* dq, void* dk, void* dv,
                       float* dgs, float* dgr, const GenericBwdWs& ws, hipStream_t st) {
  {
    ProfScope ps("gen_bwd_prep_kernel", st);
    gen_bwd_prep_kernel<IO, ST, D><<<dim3(ws.RB, dm.Hq), 256, 0, st>>>((const IO*)dO, (const ST*)sv.xs,
                                                                       (const ST*)sv.xr, sv.rs, sv.rr, gs, gr, ws.dxs,
                                                                       ws.dxr, ws.delta, ws.dgpart, dm);
  }
  if (dgs || dgr) {
    const int HD = dm.Hq * D;
    gen_dgamma_reduce_kernel<<<(HD + 255) / 256, 256, 0, st>>>(ws.dgpart, dgs, dgr, ws.RB, HD);
  }
  if (dm.nst > 0) {
    ProfScope ps("gen_scan_kernel(x2)", st);
    gen_scan_kernel<IO, IO, D, false><<<dim3(D / 16, dm.Hkv, dm.B), 256, 0, st>>>(
        (const IO*)k, (const IO*)v, ws.states, dm.T, dm.Hkv, 1, 0, dm.T - dm.W, dm.C, dm.nst, dm.phi);
    gen_scan_kernel<IO, float, D, true><<<dim3(D / 16, dm.Hkv, dm.B), 256, 0, st>>>(
        (const IO*)q, ws.dxr, ws.rstates, dm.T, dm.Hq, dm.G, dm.W, dm.T - dm.W, dm.C, dm.nst, dm.phi);
  }
  dim3 gq((dm.T + 4 * GEN_QPW - 1) / (4 * GEN_QPW), dm.Hq, dm.B);
  {
    ProfScope ps("gen_bwd_dq_kernel", st);
    gen_bwd_dq_kernel<IO, D><<<gq, 256, 0, st>>>((const IO*)q, (const IO*)k, (const IO*)v, ws.dxs, ws.dxr, ws.delta,
                                                 sv.lse, ws.states, (IO*)dq, dm);
  }
  dim3 gk((dm.T + 4 * GEN_QPW - 1) / (4 * GEN_QPW), dm.Hkv, dm.B);
  ProfScope ps("gen_bwd_dkv_kernel", st);
  gen_bwd_dkv_kernel<IO, D><<<gk, 256, 0, st>>>((const IO*)q, (const IO*)k, (const IO*)v, ws.dxs, ws.dxr, ws.delta,
                                                sv.lse, ws.rstates, (IO*)dk, (IO*)dv, dm);
}

void generic_fwd(const LayerDims& dm, int dtype, const void* q, const void* k, const void* v, const float* gs,
                 const float* gr, void* o, const SavedPtrs& sv, float* states, hipStream_t st) {
  if (dtype == 0) {
    if (dm.D == 64) launch_fwd<float, float, 64>(dm, q, k, v, gs, gr, o, sv, states, st);
    else launch_fwd<float, float, 128>(dm, q, k, v, gs, gr, o, sv, states, st);
  } else if (sv.f32) {
    if (dm.D == 64) launch_fwd<bf16_t, float, 64>(dm, q, k, v, gs, gr, o, sv, states, st);
    else launch_fwd<bf16_t, float, 128>(dm, q, k, v, gs, gr, o, sv, states, st);
  } else {
    if (dm.D == 64) launch_fwd<bf16_t, bf16_t, 64>(dm, q, k, v, gs, gr, o, sv, states, st);
    else launch_fwd<bf16_t, bf16_t, 128>(dm, q, k, v, gs, gr, o, sv, states, st);
  }
}

void generic_bwd(const LayerDims& dm, int dtype, const void* q, const void* k, const void* v, const float* gs,
                 const float* gr, const SavedPtrs& sv, const void* dO, void* dq, void* dk, void* dv, float* dgs,
                 float* dgr, const GenericBwdWs& ws, hipStream_t st) {
  if (dtype == 0) {
    if (dm.D == 64) launch_bwd<float, float, 64>(dm, q, k, v, gs, gr, sv, dO, dq, dk, dv, dgs, dgr, ws, st);
    else launch_bwd<float, float, 128>(dm, q, k, v, gs, gr, sv, dO, dq, dk, dv, dgs, dgr, ws, st);
  } else if (sv.f32) {
    if (dm.D == 64) launch_bwd<bf16_t, float, 64>(dm, q, k, v, gs, gr, sv, dO, dq, dk, dv, dgs, dgr, ws, st);
    else launch_bwd<bf16_t, float, 128>(dm, q, k, v, gs, gr, sv, dO, dq, dk, dv, dgs, dgr, ws, st);
  } else {
    if (dm.D == 64) launch_bwd<bf16_t, bf16_t, 64>(dm, q, k, v, gs, gr, sv, dO, dq, dk, dv, dgs, dgr, ws, st);
    else launch_bwd<bf16_t, bf16_t, 128>(dm, q, k, v, gs, gr, sv, dO, dq, dk, dv, dgs, dgr, ws, st);
  }
}

}  // namespace rattn
