// MFMA backward of the RAttention layer (same shape class as the MFMA forward: bf16, D = 128,
// T % 128 == 0, any W >= 8; tiles and states are laid out for W rounded up to 64, see fast_fwd.hip).
// No floating-point atomics: dq is produced by a kernel that owns query tiles, dk/dv by a kernel that
// owns key tiles (and visits the G query heads of its KV head in turn); both recompute the attention
// probabilities from the saved log-sum-exp.
//
//   RMS  : through the two RMS norms (Sec. 3.2), as the prologue of the dq kernel: dx_s, dx_r (bf16 MFMA
//          operands, also written out for the kernels that follow), delta = <dx_s, x_s>, dgamma partials
//   states: S_[j] (Eq. 2, kept by the forward pass) and the reverse-time states R_[j] = sum_{later chunks} phi(q)^T dx_r
//   dq   : transposed, lane = query:  dQ^T = scale * K^T dS^T,  dS = P .* (dP - delta),  dP^T = V dXs^T
//          linear branch: dphi(Q)^T = S dXr^T + Kf^T (M^T .* (V dXr^T)), then the softmax Jacobian of phi
//   dkv  : transposed, lane = key:   dV^T = dXs^T P + dXr^T C + R^T Kf^T,
//          dK^T = scale * Q^T dS + J_phi(Qf^T dC + R V^T)
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"
#include <type_traits>
#include <limits.h>

namespace rattn {

namespace {

struct FastBwdArgs {
  const uint16_t *q, *k, *v, *dxs, *dxr;
  const float *lse, *delta;
  const uint16_t *states, *rstates;
  uint16_t *dq, *dk, *dv;
  int B, T, Hq, Hkv, G, W, gap, nstf, nk, ntile;  // W: window rounded up to 64; true window = W - gap
  float scale, scale_log2;
  // inputs of the RMS-norm backward in the dq kernel's prologue, which fills dxs, dxr and delta above
  const uint16_t *dO, *xs, *xr;
  // ragged lengths (see split_rows in mfma.hpp): rows >= Tfull of the caller's q, k, v, dO, dq, dk, dv live in 128-row
  // tail buffers; Tc = rows per sequence of the caller's tensors.  T above is the padded length: saved tensors, the
  // workspace tensors (dxs, dxr, delta) and the states are laid out for it.
  const uint16_t *q_tail, *k_tail, *v_tail, *dO_tail;
  uint16_t *dq_tail, *dk_tail, *dv_tail;
  int Tc, Tfull;
  const float *rs, *rr, *gs, *gr;  // gains: NULL = ones
  float* dgpart;                   // gain-gradient partials [2][4 * ntile * B][Hq][128], NULL = not wanted
  float inv_d;                     // 1 / head size the RMS norms average over (1/64 for rows zero-padded from 64)
};

// ------------------------------------------------------------------------------------------------
// Sums the per-wave gain-gradient partials of the dq kernel's prologue, in a fixed order.  grid (HD / 32, 2),
// 256 threads: the work-group owns 32 consecutive (head, feature) entries of one of the two gains; thread
// (rg = tid / 8, c = tid % 8) adds every 32nd partial starting at rg for entries 4c .. 4c+3 (independent 16-byte
// loads), then the 32 sums are added in order.
__global__ __launch_bounds__(256) void dgamma_reduce_kernel(const float* __restrict__ dgpart, float* __restrict__ dgs,
                                                            float* __restrict__ dgr, int RB, int HD) {
  __shared__ float4 part[32][8];
  const int which = blockIdx.y, rg = threadIdx.x >> 3, c = threadIdx.x & 7;
  float* out = which ? dgr : dgs;
  if (!out) return;
  const int i = blockIdx.x * 32 + 4 * c;
  const float* src = dgpart + (size_t)which * RB * HD + i;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
  for (int r = rg; r < RB; r += 32) {
    const float4 x = *reinterpret_cast<const float4*>(src + (size_t)r * HD);
    s.x += x.x; s.y += x.y; s.z += x.z; s.w += x.w;
  }
  part[rg][c] = s;
  __syncthreads();
  if (rg == 0) {
    float4 t = part[0][c];
#pragma unroll
    for (int j = 1; j < 32; ++j) { const float4 x = part[j][c]; t.x += x.x; t.y += x.y; t.z += x.z; t.w += x.w; }
    *reinterpret_cast<float4*>(out + i) = t;
  }
}

// row `src` (128 bf16) re-read in accumulator layout: lane keeps features 32ft + 8*i4 + 4h + e -> x[ft*16 + 4*i4 + e];
// phi of that row (the row's other half sits in lane ^ 32).  FM_SOFTMAX64: features 64..127 (ft >= 2) are padding.
// the 16 8-byte pieces of row `src` that a lane holds in accumulator layout (piece 4 ft + i4 = features
// 32ft + 8*i4 + 4h .. +3): fetched ahead of their use, unpacked by phi_row_clayout
__device__ __forceinline__ void load_row_clayout(const uint16_t* src, int h, bf16x4_t (&raw)[16]) {
#pragma unroll
  for (int ft = 0; ft < 4; ++ft)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) raw[4 * ft + i4] = *reinterpret_cast<const bf16x4_t*>(src + 32 * ft + 8 * i4 + 4 * h);
}

template <int FM>
__device__ __forceinline__ void phi_row_clayout(const bf16x4_t (&raw)[16], float (&x)[64]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    f32x4_t f = __builtin_convertvector(raw[j], f32x4_t);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[4 * j + e] = f[e];
  }
  if (FM == FM_RELU) {
#pragma unroll
    for (int i = 0; i < 64; ++i) x[i] = fmaxf(x[i], 0.f);
    return;
  }
  constexpr int NV = FM == FM_SOFTMAX64 ? 32 : 64;
  float m = x[0];
#pragma unroll
  for (int i = 1; i < NV; ++i) m = fmaxf(m, x[i]);
  m = half_max(m);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) { x[i] = fast_exp2((x[i] - m) * LOG2E); s += x[i]; }
  s = half_sum(s);
  const float inv = 1.f / s;
#pragma unroll
  for (int i = 0; i < NV; ++i) x[i] *= inv;
#pragma unroll
  for (int i = NV; i < 64; ++i) x[i] = 0.f;
}

// acc <- f .* (acc - <acc, f>)   (softmax Jacobian applied to a gradient held in accumulator layout; padding features
// have f = 0 and come out as 0);  ReLU map: acc <- acc where the input was positive, i.e. where f = max(x, 0) > 0
template <int FM>
__device__ __forceinline__ void phi_jacobian(f32x16_t (&acc)[4], const float (&f)[64]) {
  if (FM == FM_RELU) {
#pragma unroll
    for (int ft = 0; ft < 4; ++ft)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[ft][i] = f[ft * 16 + i] > 0.f ? acc[ft][i] : 0.f;
    return;
  }
  float inner = 0.f;
#pragma unroll
  for (int ft = 0; ft < 4; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) inner += acc[ft][i] * f[ft * 16 + i];
  inner = half_sum(inner);
#pragma unroll
  for (int ft = 0; ft < 4; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[ft][i] = f[ft * 16 + i] * (acc[ft][i] - inner);
}

__device__ __forceinline__ void load_bop(const uint16_t* rowp, int h, bf16x8_t (&op)[8]) {
#pragma unroll
  for (int c = 0; c < 8; ++c) op[c] = *reinterpret_cast<const bf16x8_t*>(rowp + 16 * c + 8 * h);
}

// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void dq_subtile(const unsigned char* kt, const unsigned char* vt, int ks, int ka, int myq,
                                           int W, bool masked, float scale, float scale_log2, float lse2, float dl,
                                           const bf16x8_t (&qop)[8], const bf16x8_t (&dxsop)[8], f32x16_t (&acc)[4],
                                           int lane, const LaneOff& lo) {
  const int h = lane >> 5;
  f32x16_t s = {0}, dp = {0};
#pragma unroll
  for (int c = 0; c < 8; ++c) s = mfma32(lds_row(kt, lo, 32 * ks, c), qop[c], s);
#pragma unroll
  for (int c = 0; c < 8; ++c) dp = mfma32(lds_row(vt, lo, 32 * ks, c), dxsop[c], dp);
  // probabilities of the unmasked case; they depend on the first chain only, so they are scheduled into the
  // second chain (masked entries are zeroed afterwards, which equals masking the logits)
  float p[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) p[i] = fast_exp2(__builtin_fmaf(s[i], scale_log2, -lse2));
  // operand reads run four ahead of the matrix chains (the default schedule issues them one ahead, which
  // exposes the LDS latency once per MFMA); the exponentials go between the MFMAs of the dP chain
  __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
  }
  if (masked) {
    // in the window <=> 0 <= query - key < W: one unsigned compare per element against a per-lane base
    const unsigned dist0 = (unsigned)(myq - ka - 4 * h);
#pragma unroll
    for (int i = 0; i < 16; ++i) p[i] = (dist0 - (unsigned)(8 * (i >> 2) + (i & 3)) < (unsigned)W) ? p[i] : 0.f;
  }
  float ds[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) ds[i] = p[i] * (dp[i] - dl) * scale;
  bf16x8_t dsop[2] = {pack_bf16x8(&ds[0]), pack_bf16x8(&ds[8])};
#pragma unroll
  for (int mf = 0; mf < 2; ++mf) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) acc[dt] = mfma32(lds_trp(kt, lo, 32 * ks + 16 * mf, dt), dsop[mf], acc[dt]);
  }
}

// grid (ntile * Hq * B), 256 threads: 128 queries of one head, wave w owns 32.
// sum over the 16 lanes of a DPP row (quad butterflies, then the two mirror steps)
template <int CTRL>
__device__ __forceinline__ float dpp_get(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float sum16(float x) {
  x += dpp_get<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_get<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_get<0x141>(x);  // row_half_mirror
  x += dpp_get<0x140>(x);  // row_mirror
  return x;
}

// Backward of the two RMS norms (Sec. 3.2) for 32 consecutive query rows of one head, by one wave: 16 lanes per row,
// 8 features each, four rows per pass (row-contiguous 16-byte accesses).  With y = g * x * r, r = rsqrt(mean x^2 +
// eps):  dx = r g dy - x r^3 mean(g dy x),  dg += dy x r.  Stores d xs, d xr (bf16) and delta = rowsum(d xs * xs)
// to global memory for the later kernels and also into LDS: d xs in two 16-row pieces at `stage_s` and
// `stage_s` + 16 KB (rows 0..15 of each, swizzled row layout; the caller passes a 16-row-aligned address: these are
// exactly the LDS rows into which the same wave later loads its share of two 64-key tiles, so no other wave's
// tile load can land on rows that are still being read) and, if `stage_r` is given, d xr into rows 0..31 of that
// tile, delta into dl_stage[0..31]; the wave
// takes them from there as MFMA operands / row statistics without waiting for (or re-reading) the global stores.
// dO, x_s, x_r are read once and d xs, d xr are not read again by this kernel: their accesses are marked
// non-temporal so that they do not push the K/V tiles, which neighbouring work-groups share, out of the L2.
// GAINS: gains other than one and/or gain gradients; the wave's gradient partials (sums over its 32 rows) go to
// dgp_s / dgp_r (128 floats each) when those are given.
template <bool GAINS>
__device__ __forceinline__ void rms_bwd_rows(const FastBwdArgs& a, int hq, size_t row0_off, const uint16_t* dO_row0,
                                             size_t qstride, size_t stat0, unsigned char* stage_s, unsigned char* stage_r, float* dl_stage,
                                             float* dgp_s, float* dgp_r, int lane) {
  const int sub = lane >> 4, c = lane & 15;
  // A query tile none of whose rows has a key beyond its window (the first tiles of a sequence; every tile of a
  // causal layer, W >= T) has x_r = 0: the forward does not store it, no later kernel reads its d x_r, and neither
  // is touched here.  The caller passes `stage_r` exactly for the tiles that have a linear branch (wave-uniform).
  const bool with_r = stage_r != nullptr;
  uint16_t* dxs_w = const_cast<uint16_t*>(a.dxs);
  uint16_t* dxr_w = const_cast<uint16_t*>(a.dxr);
  float* delta_w = const_cast<float*>(a.delta);
  float g1[8], g2[8], dg1[8], dg2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    g1[e] = (GAINS && a.gs) ? a.gs[hq * 128 + 8 * c + e] : 1.f;
    g2[e] = (GAINS && a.gr) ? a.gr[hq * 128 + 8 * c + e] : 1.f;
    dg1[e] = dg2[e] = 0.f;
  }
  // All rows are requested before the first is worked on: the loads below and the stores further down go through
  // pointers the compiler cannot tell apart, so inside one loop every iteration's loads would wait behind the
  // previous iteration's stores - eight memory round trips in a row instead of one.
  bf16x8_t dy_raw[8], xs_raw[8], xr_raw[8];
  float rs_row[8], rr_row[8];
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = 4 * it + sub;
    const size_t off = row0_off + (size_t)r * qstride + 8 * c;
    dy_raw[it] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(dO_row0 + (size_t)r * qstride + 8 * c));
    xs_raw[it] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(a.xs + off));
    rs_row[it] = a.rs[stat0 + r];
    rr_row[it] = a.rr[stat0 + r];
  }
  if (with_r) {
#pragma unroll
    for (int it = 0; it < 8; ++it)
      xr_raw[it] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(
          a.xr + row0_off + (size_t)(4 * it + sub) * qstride + 8 * c));
  } else {
#pragma unroll
    for (int it = 0; it < 8; ++it) xr_raw[it] = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
  }
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = 4 * it + sub;
    const size_t off = row0_off + (size_t)r * qstride + 8 * c;
    float dy[8], xs[8], xr[8];
    unpack_bf16x8(dy_raw[it], dy);
    unpack_bf16x8(xs_raw[it], xs);
    unpack_bf16x8(xr_raw[it], xr);
    const float r_s = rs_row[it], r_r = rr_row[it];
    float m1 = 0.f, m2 = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (GAINS) {
        dg1[e] = fmaf(dy[e] * xs[e], r_s, dg1[e]);
        dg2[e] = fmaf(dy[e] * xr[e], r_r, dg2[e]);
      }
      m1 = fmaf(g1[e] * dy[e], xs[e], m1);
      m2 = fmaf(g2[e] * dy[e], xr[e], m2);
    }
    m1 = sum16(m1) * a.inv_d;
    m2 = sum16(m2) * a.inv_d;
    const float b_s = r_s * r_s * r_s * m1, b_r = r_r * r_r * r_r * m2;
    float av[8], cv[8], dl = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      av[e] = r_s * g1[e] * dy[e] - xs[e] * b_s;
      cv[e] = r_r * g2[e] * dy[e] - xr[e] * b_r;
    }
    const bf16x8_t apk = pack_bf16x8(av);
    const bf16x8_t cpk = pack_bf16x8(cv);
    // delta from d xs as the matrix cores will see it (rounded to bf16): dS = P (dP - delta) is a near-cancellation
    // for peaked rows, and dP is formed from the rounded values
    unpack_bf16x8(apk, av);
#pragma unroll
    for (int e = 0; e < 8; ++e) dl = fmaf(av[e], xs[e], dl);
    __builtin_nontemporal_store(apk, reinterpret_cast<bf16x8_t*>(dxs_w + off));
    if (with_r) __builtin_nontemporal_store(cpk, reinterpret_cast<bf16x8_t*>(dxr_w + off));
    {  // staged in two 16-row pieces, see dxs_stage_addr
      const int R = r & 15;
      *reinterpret_cast<bf16x8_t*>(stage_s + (r >> 4) * 16384 + R * ROW_BYTES + ((c ^ swz(R)) << 4)) = apk;
    }
    if (stage_r) *reinterpret_cast<bf16x8_t*>(stage_r + r * ROW_BYTES + ((c ^ swz(r)) << 4)) = cpk;
    dl = sum16(dl);
    if (c == 0) { delta_w[stat0 + r] = dl; dl_stage[r] = dl; }
  }
  if (GAINS && dgp_s) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dg1[e] += __shfl_xor(dg1[e], 16, 64); dg1[e] += __shfl_xor(dg1[e], 32, 64);
      dg2[e] += __shfl_xor(dg2[e], 16, 64); dg2[e] += __shfl_xor(dg2[e], 32, 64);
    }
    if (sub == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { dgp_s[8 * c + e] = dg1[e]; dgp_r[8 * c + e] = dg2[e]; }
    }
  }
}

// GAINS: RMS gains other than one and/or gain gradients (see rms_bwd_rows); FM: feature map (FM_* in mfma.hpp)
template <bool GAINS, int FM>
__global__ __launch_bounds__(256, 2) void bwd_dq_kernel(FastBwdArgs a) {
  __shared__ __align__(16) unsigned char smem[65536];
  __shared__ float dl_stage[128];
  const int lane = lane_id(), w = wave_id();
  const int r32 = lane & 31, h = lane >> 5;
  const LaneOff lo = make_lane_off(lane);
  const LaneOffN lon = make_lane_off_n(lane);
  const int T = a.T, W = a.W, Hq = a.Hq, Hkv = a.Hkv, G = a.G;
  const int total = gridDim.x, bid = blockIdx.x;
  int wid = (total % 8 == 0) ? (bid % 8) * (total / 8) + bid / 8 : bid;
  const int hh = wid % G; wid /= G;
  const int qt = a.ntile - 1 - wid % a.ntile; wid /= a.ntile;  // late tiles first: they see the most keys
  const int g = wid % Hkv;
  const int b = wid / Hkv;
  const int hq = g * G + hh;
  const int t0 = qt * 128;
  const size_t qstride = (size_t)Hq * 128, kstride = (size_t)Hkv * 128;
  const size_t qtile_off = ((size_t)(b * T + t0) * Hq + hq) * 128;   // in the saved / workspace tensors (padded length)
  // the caller's tensors: this query tile of q, dO, dq; 64-key tiles of k, v
  const uint16_t* q_tile = split_rows(a.q, a.q_tail, b, t0, a.Tc, a.Tfull, Hq, hq);
  const uint16_t* dO_tile = split_rows(a.dO, a.dO_tail, b, t0, a.Tc, a.Tfull, Hq, hq);
  uint16_t* dq_tile = split_rows(a.dq, a.dq_tail, b, t0, a.Tc, a.Tfull, Hq, hq);
  auto k_rows = [&](int row) { return split_rows(a.k, a.k_tail, b, row, a.Tc, a.Tfull, Hkv, g); };
  auto v_rows = [&](int row) { return split_rows(a.v, a.v_tail, b, row, a.Tc, a.Tfull, Hkv, g); };
  const int myq = t0 + 32 * w + r32;
  const size_t stat_off = (size_t)(b * Hq + hq) * T + myq;

  const int j0 = t0 - W, gap = a.gap;
  const bool has_lin = j0 > -128 || (gap > 0 && j0 == -128);
  {
    // RMS-norm backward of this wave's 32 rows first: everything below starts from d xs, d xr and delta
    float* dgp_s = nullptr;
    float* dgp_r = nullptr;
    if (GAINS && a.dgpart) {
      const int rb = ((b * a.ntile + qt) << 2) + w;  // one partial per wave: [2][4 * ntile * B][Hq][128]
      dgp_s = a.dgpart + ((size_t)rb * Hq + hq) * 128;
      dgp_r = dgp_s + (size_t)4 * a.ntile * a.B * Hq * 128;
    }
    rms_bwd_rows<GAINS>(a, hq, qtile_off + (size_t)(32 * w) * qstride, dO_tile + (size_t)(32 * w) * qstride, qstride,
                        stat_off - r32,
                        smem + 32768 + 16 * w * ROW_BYTES, has_lin ? smem + 32 * w * ROW_BYTES : nullptr,
                        dl_stage + 32 * w, dgp_s, dgp_r, lane);
  }
  // own rows, staged by this wave in the prologue: LDS executes a wave's accesses in order, and the reads below are
  // complete (lgkmcnt wait) before this wave's tile loads may overwrite the rows.  Every later tile load of wave w
  // covers rows 16w..16w+15 of a 64-key tile (or rows 32w..32w+31 of the 128-row state tile): the staged d xs rows
  // sit in rows 16w..16w+15 of the two V tiles at 32 KB and 48 KB, the staged d xr rows in rows 32w..32w+31 of the
  // tile at 0, so a wave only ever overwrites its own staging rows.
  bf16x8_t dxsop[8];
  {
    const int R = 16 * w + (r32 & 15);  // query row r32 of this wave sits in row R of piece r32 / 16
    const unsigned char* rowp = smem + 32768 + (r32 >> 4) * 16384 + R * ROW_BYTES;
#pragma unroll
    for (int c = 0; c < 8; ++c) dxsop[c] = *reinterpret_cast<const bf16x8_t*>(rowp + (((2 * c + h) ^ swz(R)) << 4));
  }
  const float dl = dl_stage[32 * w + r32];
  f32x16_t acc[4] = {{0}, {0}, {0}, {0}};

  // ---- linear branch: d phi(q)
  // Tiles and states are laid out for the window rounded up to 64 (W); with gap = W - true window > 0 a query
  // sees key_local <= q_local + gap of the chunk that starts at j0 = t0 - W, i.e. up to 64 keys past the two
  // 64-key tiles of the aligned layout (a third tile, handled after them), and the query tile at j0 = -128
  // reaches keys only through that third tile.
  if (has_lin) {
    const bool has_state = j0 >= 0, has_res = j0 > -128;
    const int u_hi = w + ((31 + gap) >> 5);
    bf16x8_t dxrop[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) dxrop[c] = lds_row(smem, lo, 32 * w, c);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the staged rows are in registers
    // key sub-tile u (keys j0 + 32u .. +31): dC = V dXr^T, masked, then d phi(q)^T += phi(K)^T dC
    auto intra_unit = [&](const unsigned char* kt, const unsigned char* vt, int ks, int u) {
      f32x16_t c = {0};
#pragma unroll
      for (int kd = 0; kd < 8; ++kd) c = mfma32(lds_row(vt, lo, 32 * ks, kd), dxrop[kd], c);
      float cv[16];
      if (32 * u + 31 > 32 * w + gap) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key_local = 32 * u + 8 * (i >> 2) + 4 * h + (i & 3);
          cv[i] = key_local > 32 * w + r32 + gap ? 0.f : c[i];
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) cv[i] = c[i];
      }
      bf16x8_t cop[2] = {pack_bf16x8(&cv[0]), pack_bf16x8(&cv[8])};
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
#pragma unroll
        for (int ft = 0; ft < 4; ++ft) acc[ft] = mfma32(lds_trp(kt, lo, 32 * ks + 16 * mf, ft), cop[mf], acc[ft]);
      }
    };
    if (has_res) {
      if (has_state) {
        const uint16_t* sbase = a.states + ((size_t)(b * Hkv + g) * a.nstf + j0 / 128) * 16384;
        tile_load_async<8>(sbase, 128, smem, w * 8, lane);
        tile_load_async<4>(v_rows(j0), kstride, smem + 32768, w * 4, lane);
      }
      tile_load_async<4>(v_rows(j0 + 64), kstride, smem + 49152, w * 4, lane);
      wait_vmem();
      __syncthreads();
      if (has_state) {
#pragma unroll
        for (int kd = 0; kd < 8; ++kd) {
#pragma unroll
          for (int ft = 0; ft < 4; ++ft) acc[ft] = mfma32(lds_trn(smem, lon, 16 * kd, ft), dxrop[kd], acc[ft]);
        }
      }
      __syncthreads();
      if (has_state) tile_load_async<4>(k_rows(j0), kstride, smem, w * 4, lane);
      tile_load_async<4>(k_rows(j0 + 64), kstride, smem + 16384, w * 4, lane);
      wait_vmem();
      __syncthreads();
      if (has_state) phi_tile_inplace<FM>(smem, 128);
      else phi_tile_inplace<FM>(smem + 16384, 64);
      __syncthreads();
      for (int u = has_state ? 0 : 2; u <= min(3, u_hi); ++u)
        intra_unit(smem + (u >> 1) * 16384, smem + 32768 + (u >> 1) * 16384, u & 1, u);
    }
    __syncthreads();
    if (gap > 0) {
      tile_load_async<4>(k_rows(j0 + 128), kstride, smem, w * 4, lane);
      tile_load_async<4>(v_rows(j0 + 128), kstride, smem + 32768, w * 4, lane);
      wait_vmem();
      __syncthreads();
      phi_tile_inplace<FM>(smem, 64);
      __syncthreads();
      for (int u = 4; u <= min(5, u_hi); ++u) intra_unit(smem, smem + 32768, u & 1, u);
      __syncthreads();
    }
  }

  // ---- softmax branch
  // The first key tile and the work-group's q tile are requested together: q goes into the two tile buffers the
  // key sweep does not need yet (rows 0..63 and 64..127), and every wave takes its own rows from there in both of the
  // layouts it needs, instead of two more round trips to global memory for row pieces.
  if (!has_lin) __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the staged rows are in registers
  const float lse2 = a.lse[stat_off] * LOG2E;
  const int kt_lo = max(0, t0 - W);
  const int ntiles = (t0 + 128 - kt_lo) / 64;
  {
    const int kt0 = kt_lo + 64 * (ntiles - 1);
    tile_load_async<4>(k_rows(kt0), kstride, smem, w * 4, lane);
    tile_load_async<4>(v_rows(kt0), kstride, smem + 32768, w * 4, lane);
    tile_load_async<4>(q_tile, qstride, smem + 16384, w * 4, lane);
    tile_load_async<4>(q_tile + (size_t)64 * qstride, qstride, smem + 49152, w * 4, lane);
    wait_vmem();
    __syncthreads();
  }
  bf16x8_t qop[8];
  {
    const unsigned char* qhalf = smem + ((w >> 1) ? 49152 : 16384);
    const int R0 = 32 * (w & 1);
    if (has_lin) {  // phi(q) and its Jacobian close the linear branch
      const int row = R0 + r32;
      const unsigned char* rowp = qhalf + row * ROW_BYTES + 8 * h;
      bf16x4_t qraw[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) qraw[j] = *reinterpret_cast<const bf16x4_t*>(rowp + ((j ^ swz(row)) << 4));
      float qf[64];
      phi_row_clayout<FM>(qraw, qf);
      phi_jacobian<FM>(acc, qf);
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) qop[c] = lds_row(qhalf, lo, R0, c);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __syncthreads();  // the sweep's second tile load reuses the q buffers
  }
  const int qa = t0 + 32 * w, qb = qa + 31;
  const DmaLane dma_lane = make_dma_lane(lane, kstride);
  const int Wm = W - gap;  // the true window: element masks and sub-tile skipping
  // one key tile; the buffer index is a compile-time constant so that every LDS address of the sub-tile code is a
  // per-lane register plus an immediate (the loop below is unrolled by two for that)
  auto tile_step = [&](int n, auto cur_c) {
    constexpr int cur = decltype(cur_c)::value;
    const int it = ntiles - 1 - n;
    if (n + 1 < ntiles) {
      const int ktn = kt_lo + 64 * (it - 1);
      tile_load_async_s<4>(k_rows(ktn), kstride, smem + (cur ^ 1) * 16384, w * 4, dma_lane);
      tile_load_async_s<4>(v_rows(ktn), kstride, smem + 32768 + (cur ^ 1) * 16384, w * 4, dma_lane);
    }
    const unsigned char* kt = smem + cur * 16384;
    const unsigned char* vt = smem + 32768 + cur * 16384;
    const int kt0 = kt_lo + 64 * it;
#pragma unroll
    for (int ks = 1; ks >= 0; --ks) {
      const int ka = kt0 + 32 * ks;
      const bool need = ka <= qb && ka + 31 >= qa - Wm + 1;
      if (need) {
        const bool full = ka + 31 <= qa && ka >= qb - Wm + 1;
        dq_subtile(kt, vt, ks, ka, myq, Wm, !full, a.scale, a.scale_log2, lse2, dl, qop, dxsop, acc, lane, lo);
      }
    }
    wait_vmem();
    __syncthreads();
  };
  {
    int n = 0;
    for (; n + 1 < ntiles; n += 2) {
      tile_step(n, std::integral_constant<int, 0>{});
      tile_step(n + 1, std::integral_constant<int, 1>{});
    }
    if (n < ntiles) tile_step(n, std::integral_constant<int, 0>{});
  }
  float vals[4][16];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) vals[dt][i] = acc[dt][i];
  store_tile_transposed(smem, vals, dq_tile, qstride, w, lane);
}

// ------------------------------------------------------------------------------------------------
// phi in place on the first `nrows` rows of an LDS tile with 512 threads: four threads per row, 32 elements each
// (FM_SOFTMAX64: the two threads on features 64..127 leave the padding zeros alone)
template <int FM>
__device__ __forceinline__ void phi_tile_inplace_512(unsigned char* tile, int nrows) {
  const int row = threadIdx.x >> 2, part = threadIdx.x & 3;
  if (row < nrows) {
    float x[32];
    unsigned char* rp = tile + row * ROW_BYTES;
    const int sw = swz(row);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      unpack_bf16x8(*reinterpret_cast<const bf16x8_t*>(rp + (((4 * part + j) ^ sw) << 4)), &x[8 * j]);
    if (FM == FM_RELU) {
#pragma unroll
      for (int i = 0; i < 32; ++i) x[i] = fmaxf(x[i], 0.f);
    } else {
      float m = x[0];
#pragma unroll
      for (int i = 1; i < 32; ++i) m = fmaxf(m, x[i]);
      m = fmaxf(m, __shfl_xor(m, 1, 64));
      if (FM == FM_SOFTMAX) m = fmaxf(m, __shfl_xor(m, 2, 64));
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 32; ++i) { x[i] = fast_exp2((x[i] - m) * LOG2E); sum += x[i]; }
      sum += __shfl_xor(sum, 1, 64);
      if (FM == FM_SOFTMAX) sum += __shfl_xor(sum, 2, 64);
      const float inv = 1.f / sum;
#pragma unroll
      for (int i = 0; i < 32; ++i) x[i] *= inv;
    }
    if (!(FM == FM_SOFTMAX64 && part >= 2)) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<bf16x8_t*>(rp + (((4 * part + j) ^ sw) << 4)) = pack_bf16x8(&x[8 * j]);
    }
  }
}

// LDS map of the dk/dv kernel: three 32 KB slots, each a 64-row q tile followed by a 64-row dx tile; 32 KB for the
// probabilities handed from the V-role to the K-role waves; per slot the 64 log-sum-exp and 64 delta values of
// its rows.  The linear branch uses the same space as two buffers of one 128-row q tile and one 128-row dx tile
// each: A = slots 0-1, B = slot 2 + the hand-over area (which first receives the reverse-state tile).
constexpr int DKV_SLOT = 32768, DKV_PEX_OFF = 98304, DKV_STAT_OFF = 131072;
constexpr int DKV_LDS_BYTES = DKV_STAT_OFF + 3 * 2048;

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// grid (ntile * Hkv * B), 512 threads: 128 keys of one KV head.  Waves w and 7-w both work on key block w
// (lane = key) with complementary roles, so each keeps only one 128 x 32 accumulator and one set of operand
// rows and two waves (w and w+4, one of each role) fit on a SIMD:
//   V-role (waves 0-3): S^T = Q K^T -> P (also written to LDS, fp32),  dV^T += dXs^T P;
//                       linear branch: C = phi(Q) phi(K)^T (masked),   dV^T += dXr^T C + R-state rows * phi(K)
//   K-role (waves 4-7): dP = dXs V^T, then dS = P .* (dP - delta) * scale with the P of its partner,
//                       dK^T += Q^T dS;  linear branch: dC = dXr V^T (masked), dphi(K)^T += phi(Q)^T dC + R V^T,
//                       softmax Jacobian of phi before the softmax-branch terms are added.
// Per 32-query sub-tile one work-group barrier hands P over (LDS buffer alternates with the sub-tile parity).
// Query tiles run through three LDS buffers: tile s+2 is requested right after the first barrier of step s
// (every wave has then left tile s-1, whose buffer it takes) and each wave waits for its share of tile s+1
// before the second barrier of step s, so no further barrier is needed.  The loop has no other vector-memory
// operation (row statistics arrive with the tiles), which is what makes the explicit counter waits exact.
template <int FM>
__global__ __launch_bounds__(512) void bwd_dkv_kernel(FastBwdArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* pex = smem + DKV_PEX_OFF;
  const int lane = lane_id(), w8 = wave_id();
  const bool krole = w8 >= 4;
  // key block of the wave: the K-role takes them in reverse, so that in the linear branch, where block j pairs with
  // 4 - j query sub-tiles, the two waves of every SIMD (w8 and w8 + 4) carry five sub-tiles between them
  const int w = krole ? 7 - w8 : w8;
  const int r32 = lane & 31, h = lane >> 5;
  const LaneOff lo = make_lane_off(lane);
  const int T = a.T, W = a.W, Hq = a.Hq, Hkv = a.Hkv, G = a.G;
  const int total = gridDim.x, bid = blockIdx.x;
  int wid = (total % 8 == 0) ? (bid % 8) * (total / 8) + bid / 8 : bid;
  const int kti = wid % a.ntile; wid /= a.ntile;
  const int g = wid % Hkv;
  const int b = wid / Hkv;
  const int s0 = kti * 128;
  const int Tp = T - W;
  const size_t qstride = (size_t)Hq * 128, kstride = (size_t)Hkv * 128;
  // this key tile in the caller's k, v, dk, dv (the last, partial tile of a ragged length lives in the tail buffers)
  const size_t myrow = (size_t)(32 * w + r32) * kstride;
  const uint16_t* k_myrow = split_rows(a.k, a.k_tail, b, s0, a.Tc, a.Tfull, Hkv, g) + myrow;
  const uint16_t* v_myrow = split_rows(a.v, a.v_tail, b, s0, a.Tc, a.Tfull, Hkv, g) + myrow;
  const int mykey = s0 + 32 * w + r32;

  bf16x8_t xop[8];  // V-role: K rows (phi(K) rows during the linear branch); K-role: V rows
  load_bop(krole ? v_myrow : k_myrow, h, xop);
  f32x16_t acc[4] = {{0}, {0}, {0}, {0}};  // V-role: dV^T; K-role: dK^T
  // what each role needs of its K rows right after the linear branch, fetched now so that no global load sits on the
  // path between the two branches: the K-role the row in accumulator layout (softmax Jacobian), the V-role a copy of
  // the raw rows (xop holds phi(K) meanwhile)
  // (one register set for both roles: 8 x 16 bytes)
  bf16x8_t kkeep[8];

  // ---- request machinery of the softmax branch (query tiles of 64 rows from s0 up to the last row that still
  // sees these keys); defined first because the linear branch already requests the first tiles
  const int n_qt = (min(s0 + 128 + W, T) - s0) / 64;
  const int nsteps = G * n_qt;
  const int ka = s0 + 32 * w;
  // per-lane part of the tile addresses (swizzled 16-byte chunk of rows 8*w8 + lane/16 and +4), computed once
  const int ir0 = 8 * w8 + (lane >> 4), ir1 = ir0 + 4, ip = lane & 15;
  const unsigned lane_g0 = (unsigned)(((size_t)ir0 * qstride + ((ip ^ swz(ir0)) << 3)) * 2);  // bytes
  const unsigned lane_g1 = (unsigned)(((size_t)ir1 * qstride + ((ip ^ swz(ir1)) << 3)) * 2);
  const unsigned lds_q = (unsigned)(size_t)RATTN_LDS(smem) + w8 * 2048;
  const unsigned lds_st = (unsigned)(size_t)RATTN_LDS(smem + DKV_STAT_OFF) + (krole ? 1024 : 0);
  const float* stat_base = (krole ? a.delta : a.lse) + (size_t)(b * Hq + g * G) * T + s0;  // lane adds 16 * ip bytes
  const size_t tile_g = ((size_t)(b * T + s0) * Hq + g * G) * 128;   // workspace tensors (padded length)
  int is_h = 0, is_n = 0, is_buf = 0;  // head, tile and slot of the next tile to request
  auto issue = [&]() {
    const size_t qoff = tile_g + (size_t)is_n * 64 * qstride + (size_t)is_h * 128;
    const uint16_t* qsrc = split_rows(a.q, a.q_tail, b, s0 + 64 * is_n, a.Tc, a.Tfull, Hq, g * G + is_h);
    dma16s(qsrc, lane_g0, lds_q + is_buf * DKV_SLOT);
    dma16s(qsrc, lane_g1, lds_q + is_buf * DKV_SLOT + 1024);
    dma16s(a.dxs + qoff, lane_g0, lds_q + is_buf * DKV_SLOT + 16384);
    dma16s(a.dxs + qoff, lane_g1, lds_q + is_buf * DKV_SLOT + 16384 + 1024);
    if (w == 0)  // one wave of each role: the row statistics that role consumes (lanes 16.. fetch duplicates)
      dma16s(stat_base + (size_t)is_h * T + 64 * is_n, 16 * ip, lds_st + is_buf * 2048);
    if (++is_n == n_qt) { is_n = 0; ++is_h; }
    if (++is_buf == 3) is_buf = 0;
  };
  int buf = 0, issued = 0;  // slot of the first softmax-branch tile, tiles requested so far

  // ---- linear branch
  // Key s pairs with the queries t >= s + (true window).  In the aligned layout (W) those of this key tile are
  // the "head" rows t = s0 + W + [0, nq) of every query head, masked to q_local >= key_local, plus everything
  // later through the reverse state.  With gap = W - true window > 0 a key also pairs with up to `gap` earlier
  // queries, q_local >= key_local - gap: they lie in the 64 rows before the head rows, which are run as a
  // second (first) pass per head.  A pass = 64 or 128 query rows of one head, q_local of its first row = qb0.
  const int gap = a.gap;
  const bool has_main = s0 < Tp;
  const bool has_pre = gap > 0 && s0 <= Tp;
  if (has_main || has_pre) {
    const int nq = has_main ? min(128, Tp - s0) : 0;  // head rows
    const int np = (has_pre ? 1 : 0) + (has_main ? 1 : 0), NV = G * np;
    if (krole) {
      bf16x4_t kraw[16];
      load_row_clayout(k_myrow, h, kraw);
#pragma unroll
      for (int j = 0; j < 8; ++j) kkeep[j] = __builtin_shufflevector(kraw[2 * j], kraw[2 * j + 1], 0, 1, 2, 3, 4, 5, 6, 7);
    }
    unsigned char* const qA = smem;
    unsigned char* const dA = smem + 32768;
    unsigned char* const qB = smem + 65536;
    unsigned char* const dB = smem + DKV_PEX_OFF;
    auto pass_is_pre = [&](int vh) { return has_pre && (vh % np) == 0; };
    auto issue_pass = [&](int vh, unsigned char* qb, unsigned char* db) {
      const bool pre = pass_is_pre(vh);
      const int row0 = s0 + W - (pre ? 64 : 0), nrow = pre ? 64 : nq;
      const size_t qoff = ((size_t)(b * T + row0) * Hq + g * G + vh / np) * 128;   // workspace tensor (padded length)
      tile_load_async<2>(split_rows(a.q, a.q_tail, b, row0, a.Tc, a.Tfull, Hq, g * G + vh / np), qstride, qb, w8 * 2, lane);
      tile_load_async<2>(a.dxr + qoff, qstride, db, w8 * 2, lane);
      if (nrow == 128) {
        // rows 64..127 of the pass: their own source (row0 is a multiple of 64, the half tile may be the ragged tail);
        // the loader adds 64 row strides for these blocks, so the base is given 64 rows back (never dereferenced there)
        const uint16_t* q64 = split_rows(a.q, a.q_tail, b, row0 + 64, a.Tc, a.Tfull, Hq, g * G + vh / np);
        tile_load_async<2>(q64 - (size_t)64 * qstride, qstride, qb, 16 + w8 * 2, lane);
        tile_load_async<2>(a.dxr + qoff, qstride, db, 16 + w8 * 2, lane);
      }
    };
    if (has_main) {
      const uint16_t* rbase = a.rstates + ((size_t)(b * Hkv + g) * a.nk + kti) * 16384;
      tile_load_async<4>(rbase, 128, dB, w8 * 4, lane);
    }
    issue_pass(0, qA, dA);
    if (!krole) {  // phi of the own K rows while the first tiles are on their way
      float x[64];
#pragma unroll
      for (int c = 0; c < 8; ++c) { kkeep[c] = xop[c]; unpack_bf16x8(xop[c], &x[8 * c]); }
      phi_rows<FM>(x, xop);
    }
    wait_vmem();
    __syncthreads();
    if (has_main) {
      if (!krole) {
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
          for (int t = 0; t < 4; ++t) acc[t] = mfma32(lds_row(dB, lo, 32 * t, c), xop[c], acc[t]);
      } else {
        const LaneOffN lon = make_lane_off_n(lane);
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
          for (int t = 0; t < 4; ++t) acc[t] = mfma32(lds_trn(dB, lon, 16 * c, t), xop[c], acc[t]);
      }
    }
    __syncthreads();  // buffer B is free again
    for (int vh = 0; vh < NV; ++vh) {
      const bool in_a = !(vh & 1);
      unsigned char* const qb = in_a ? qA : qB;
      unsigned char* const db = in_a ? dA : dB;
      // while this pass is worked on, the other buffer receives the next one, or after the last pass the
      // first query tiles of the softmax branch (slot 2 if buffer B is the free one, else slots 0 and 1)
      if (vh + 1 < NV) {
        issue_pass(vh + 1, in_a ? qB : qA, in_a ? dB : dA);
      } else if (in_a) {
        is_buf = buf = 2;
        issue();
        issued = 1;
      } else {
        issue();
        issued = 1;
        if (nsteps > 1) { issue(); issued = 2; }
      }
      const bool pre = pass_is_pre(vh);
      const int nrow = pre ? 64 : nq, qb0 = pre ? -64 : 0;
      phi_tile_inplace_512<FM>(qb, nrow);
      __syncthreads();
      const unsigned char* mine = krole ? db : qb;    // rows contracted with xop
      const unsigned char* other = krole ? qb : db;   // rows accumulated into acc
      for (int u = 0; u < nrow / 32; ++u) {
        const int ql0 = qb0 + 32 * u;                  // q_local of the sub-tile's first row
        if (32 * w > ql0 + 31 + gap) continue;         // no pair of this key block and sub-tile
        f32x16_t c = {0};
#pragma unroll
        for (int e = 0; e < 8; ++e) c = mfma32(lds_row(mine, lo, 32 * u, e), xop[e], c);
        float cv[16];
        if (32 * w + 31 > ql0 + gap) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int q_local = ql0 + 8 * (i >> 2) + 4 * h + (i & 3);
            cv[i] = 32 * w + r32 > q_local + gap ? 0.f : c[i];
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) cv[i] = c[i];
        }
        const bf16x8_t cop[2] = {pack_bf16x8(&cv[0]), pack_bf16x8(&cv[8])};
#pragma unroll
        for (int mf = 0; mf < 2; ++mf)
#pragma unroll
          for (int t = 0; t < 4; ++t) acc[t] = mfma32(lds_trp(other, lo, 32 * u + 16 * mf, t), cop[mf], acc[t]);
      }
      wait_vmem();
      __syncthreads();  // what was requested above has landed, and everyone is done with this buffer
    }
    if (krole) {
      float kf[64];
      bf16x4_t kraw[16];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        kraw[2 * j] = __builtin_shufflevector(kkeep[j], kkeep[j], 0, 1, 2, 3);
        kraw[2 * j + 1] = __builtin_shufflevector(kkeep[j], kkeep[j], 4, 5, 6, 7);
      }
      phi_row_clayout<FM>(kraw, kf);
      phi_jacobian<FM>(acc, kf);
    } else {
#pragma unroll
      for (int c = 0; c < 8; ++c) xop[c] = kkeep[c];
    }
  }

  // ---- softmax branch
  const int Wm = W - gap;  // the true window: element masks and sub-tile skipping
  if (issued == 0) {
    issue();
    if (nsteps > 1) issue();
    wait_vmem();
    __syncthreads();
  } else if (issued == 1 && nsteps > 1) {
    issue();  // tile 0 is already visible; tile 1 has all of step 0 to arrive
  }
  // The loop exists once per role (the role is fixed per wave): with the role a compile-time constant the code between
  // two barriers has no role branches in it, which the instruction scheduler needs to overlap a chain with its reads.
  auto tile_loop = [&](auto role) {
    constexpr bool KR = decltype(role)::value;
    int n = 0;
    for (int step = 0; step < nsteps; ++step, buf = buf == 2 ? 0 : buf + 1, n = n + 1 == n_qt ? 0 : n + 1) {
      const unsigned char* qtile = smem + buf * DKV_SLOT;
      const unsigned char* dxt = qtile + 16384;
      const float* stat_lds = reinterpret_cast<const float*>(smem + DKV_STAT_OFF + buf * 2048 + (KR ? 1024 : 0));
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) {
        const int qa = s0 + 64 * n + 32 * qs;
        const bool need = qa + 31 >= ka && qa <= ka + 31 + Wm - 1;
        const bool full = qa >= ka + 31 && qa + 31 <= ka + Wm - 1;
        f32x4_t* px = reinterpret_cast<f32x4_t*>(pex + (w * 2 + qs) * 4096 + lane * 16);  // [i4][lane] x 16 bytes
        f32x16_t s = {0};
        float stat[16];
        if (need) {
          const unsigned char* rows = KR ? dxt : qtile;
#pragma unroll
          for (int c = 0; c < 8; ++c) s = mfma32(lds_row(rows, lo, 32 * qs, c), xop[c], s);
          __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);  // operand reads run four ahead of the chain
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const f32x4_t f = *reinterpret_cast<const f32x4_t*>(stat_lds + 32 * qs + 8 * i4 + 4 * h);
            stat[4 * i4] = f[0]; stat[4 * i4 + 1] = f[1]; stat[4 * i4 + 2] = f[2]; stat[4 * i4 + 3] = f[3];
          }
          if (!KR) {
            if (!full) {
              const unsigned dist0 = (unsigned)(qa + 4 * h - mykey);  // 0 <= query - key < W, one compare per element
#pragma unroll
              for (int i = 0; i < 16; ++i)
                s[i] = (dist0 + (unsigned)(8 * (i >> 2) + (i & 3)) < (unsigned)Wm) ? s[i] : -INFINITY;
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) s[i] = fast_exp2(__builtin_fmaf(s[i], a.scale_log2, -stat[i] * LOG2E));
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) px[i4 * 64] = f32x4_t{s[4 * i4], s[4 * i4 + 1], s[4 * i4 + 2], s[4 * i4 + 3]};
          }
        }
        if (qs == 1) {  // this wave's share of tile step+1 has landed (tile step+2 may still be in flight)
          if (step + 2 < nsteps) {
            if (w == 0) wait_vmcnt<5>();
            else wait_vmcnt<4>();
          } else {
            wait_vmcnt<0>();
          }
        }
        __syncthreads();  // P of this sub-tile is in LDS
        if (qs == 0 && step + 2 < nsteps) issue();
        if (need) {
          float x[16];
          if (!KR) {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = s[i];
          } else {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              const f32x4_t pv = px[i4 * 64];
#pragma unroll
              for (int e = 0; e < 4; ++e) x[4 * i4 + e] = pv[e] * (s[4 * i4 + e] - stat[4 * i4 + e]) * a.scale;
            }
          }
          const bf16x8_t xo[2] = {pack_bf16x8(&x[0]), pack_bf16x8(&x[8])};
          const unsigned char* cols = KR ? qtile : dxt;
#pragma unroll
          for (int mf = 0; mf < 2; ++mf)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) acc[dt] = mfma32(lds_trp(cols, lo, 32 * qs + 16 * mf, dt), xo[mf], acc[dt]);
        }
      }
    }
  };
  if (krole) tile_loop(std::true_type{});
  else tile_loop(std::false_type{});
  __syncthreads();
  // ---- dV^T (V-role) and dK^T (K-role) leave through LDS as two row-major tiles
  {
    unsigned char* tile = smem + (krole ? 32768 : 0);
    const int row = 32 * w + r32;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        f32x4_t f = {acc[dt][4 * i4], acc[dt][4 * i4 + 1], acc[dt][4 * i4 + 2], acc[dt][4 * i4 + 3]};
        const int c = 4 * dt + i4;
        *reinterpret_cast<bf16x4_t*>(tile + row * ROW_BYTES + ((c ^ swz(row)) << 4) + 8 * h) =
            __builtin_convertvector(f, bf16x4_t);
      }
    __syncthreads();
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int id = tid + 512 * i;
      const int which = id >> 11, r = (id >> 4) & 127, pch = id & 15;
      const int c = pch ^ swz(r);
      const u32x4_t val = *reinterpret_cast<const u32x4_t*>(smem + which * 32768 + r * ROW_BYTES + (pch << 4));
      uint16_t* dst = which ? split_rows(a.dk, a.dk_tail, b, s0, a.Tc, a.Tfull, Hkv, g)
                            : split_rows(a.dv, a.dv_tail, b, s0, a.Tc, a.Tfull, Hkv, g);
      __builtin_nontemporal_store(val, reinterpret_cast<u32x4_t*>(dst + (size_t)r * kstride + c * 8));
    }
  }
}

}  // namespace

void fast_bwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs, const float* gr,
              const SavedPtrs& sv, const void* dO, void* dq, void* dk, void* dv, float* dgs, float* dgr,
              const FastBwdWs& ws, hipStream_t st, const RaggedTails* tails) {
  const FastBwdPlan pl = fast_bwd_plan(dm);
  // The RMS-norm backward runs as the prologue of the dq kernel (each wave on its own rows); the variant with
  // gains also leaves per-wave partials of the gain gradients, summed afterwards in a fixed order.
  const bool gains = gs || gr || dgs || dgr;
  FastBwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.dxs = (const uint16_t*)ws.dxs; a.dxr = (const uint16_t*)ws.dxr;
  a.lse = sv.lse; a.delta = ws.delta;
  // chunk states of the forward pass: kept in `saved`, or (state policy "rebuild") built again here from k and v
  // (or, with a state stride, every m-th kept and the ones in between built again from those)
  const bool all_kept = sv.states && sv.state_stride <= 1;
  if (!all_kept && pl.fwd.nstf > 0)
    rla_forward_states(dm, pl.fwd, k, v, ws.U, ws.states, st, nullptr, tails, nullptr,
                       sv.state_stride > 1 ? sv.states : nullptr, sv.state_stride);
  a.states = (const uint16_t*)(all_kept ? sv.states : ws.states); a.rstates = (const uint16_t*)ws.rstates;
  a.dq = (uint16_t*)dq; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv;
  a.q_tail = tails ? (const uint16_t*)tails->q : nullptr; a.k_tail = tails ? (const uint16_t*)tails->k : nullptr;
  a.v_tail = tails ? (const uint16_t*)tails->v : nullptr; a.dO_tail = tails ? (const uint16_t*)tails->dO : nullptr;
  a.dq_tail = tails ? (uint16_t*)tails->dq : nullptr; a.dk_tail = tails ? (uint16_t*)tails->dk : nullptr;
  a.dv_tail = tails ? (uint16_t*)tails->dv : nullptr;
  a.Tc = tails ? tails->Tc : dm.T;
  a.Tfull = tails ? tails->Tc / 128 * 128 : INT_MAX;
  a.B = dm.B; a.T = dm.T; a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.G = dm.G; a.W = pl.fwd.W; a.gap = pl.fwd.gap;
  a.nstf = pl.fwd.nstf; a.nk = pl.nk; a.ntile = dm.T / 128;
  a.scale = dm.scale; a.scale_log2 = dm.scale * LOG2E;
  a.dO = (const uint16_t*)dO; a.xs = (const uint16_t*)sv.xs; a.xr = (const uint16_t*)sv.xr;
  a.rs = sv.rs; a.rr = sv.rr; a.gs = gs; a.gr = gr;
  a.dgpart = (dgs || dgr) ? ws.dgpart : nullptr;
  a.inv_d = 1.f / (float)dm.Dv;
  // (softmax and ReLU maps only: with the identity map the host layer sends every call that keeps `saved` to the
  // general kernels, see make_layout)
  const int fm = feature_map_variant(dm);
  {
    ProfScope ps("bwd_dq_kernel", st);
    const dim3 grid(a.ntile * dm.Hq * dm.B);
#define RATTN_DQ_LAUNCH(FM_)                                                   \
  do {                                                                         \
    if (gains) bwd_dq_kernel<true, FM_><<<grid, 256, 0, st>>>(a);              \
    else bwd_dq_kernel<false, FM_><<<grid, 256, 0, st>>>(a);                   \
  } while (0)
    switch (fm) {
      case FM_RELU: RATTN_DQ_LAUNCH(FM_RELU); break;
      case FM_SOFTMAX64: RATTN_DQ_LAUNCH(FM_SOFTMAX64); break;
      default: RATTN_DQ_LAUNCH(FM_SOFTMAX); break;
    }
#undef RATTN_DQ_LAUNCH
  }
  if (dgs || dgr) {
    const int HD = dm.Hq * 128;
    ProfScope ps("dgamma_reduce_kernel", st);
    dgamma_reduce_kernel<<<dim3(HD / 32, 2), 256, 0, st>>>(ws.dgpart, dgs, dgr, pl.RB, HD);
  }
  rla_reverse_states(dm, pl, q, ws.dxr, ws.U, ws.rstates, st, tails);
  // the dk/dv kernel needs more LDS than a launch gets by default: raised once per instantiation
  static const bool lds_attr = [] {
    const void* fns[] = {reinterpret_cast<const void*>(bwd_dkv_kernel<FM_SOFTMAX>),
                         reinterpret_cast<const void*>(bwd_dkv_kernel<FM_RELU>),
                         reinterpret_cast<const void*>(bwd_dkv_kernel<FM_SOFTMAX64>)};
    bool ok = true;
    for (const void* f : fns) ok &= hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, DKV_LDS_BYTES) == hipSuccess;
    return ok;
  }();
  (void)lds_attr;
  ProfScope ps("bwd_dkv_kernel", st);
  const dim3 kgrid(a.ntile * dm.Hkv * dm.B);
  switch (fm) {
    case FM_RELU: bwd_dkv_kernel<FM_RELU><<<kgrid, 512, DKV_LDS_BYTES, st>>>(a); break;
    case FM_SOFTMAX64: bwd_dkv_kernel<FM_SOFTMAX64><<<kgrid, 512, DKV_LDS_BYTES, st>>>(a); break;
    default: bwd_dkv_kernel<FM_SOFTMAX><<<kgrid, 512, DKV_LDS_BYTES, st>>>(a); break;
  }
}

}  // namespace rattn
