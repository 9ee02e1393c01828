// MFMA forward of the RAttention layer for bf16, D = 128, T % 128 == 0, any window W >= 8.
// Tiles, chunk states and loop ranges are laid out for the window rounded up to a multiple of 64 (`W` in the
// kernel arguments); `gap` = that minus the true window (0..63) enters only the element masks and, in the linear
// branch, the reach of the intra-chunk part (queries see `gap` more keys than the aligned layout gives them).
//
// One work-group (4 waves) owns 128 consecutive queries of one head; wave w owns 32 of them.
// Everything is computed TRANSPOSED so that a lane always owns one query (column) of the MFMA
// results and all row statistics are lane-local (plus one exchange with lane^32):
//   softmax branch (Sec. 2.1):  S^T = K Q^T  ->  online softmax  ->  O^T += V^T P^T
//   linear branch (Eqs. 2-4) :  X^T = St Qf^T  +  V^T (M^T .* (Kf Qf^T)),  St = S_[j]^T (bf16, from the
//                               state pre-pass), Qf/Kf = phi(Q)/phi(K) computed on the operand registers
//   combination (Sec. 3.2)   :  o = gs * x_s * r_s + gr * x_r * r_r, transposed through LDS for
//                               coalesced stores
// K/V tiles (64 keys) stream through a double buffer in LDS with direct-to-LDS loads; the softmax branch
// walks its key tiles from the diagonal downwards (every row's running maximum is finite from the start),
// then the linear branch runs on the two lowest tiles, which are still resident; the normalised softmax-branch
// result stays in fp32 registers meanwhile, so the output is rounded to bf16 once.
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"
#include <limits.h>

namespace rattn {

namespace {

struct FastFwdArgs {
  const uint16_t *q, *k, *v;
  const float *gs, *gr;
  uint16_t *o, *xs_out, *xr_out;
  // ragged lengths (see split_rows): rows >= Tfull of q, k, v, o live in 128-row tail buffers; Tcq / Tck = rows per
  // sequence of the caller's q, o / k, v tensors (the saved tensors and the states are laid out for the padded T)
  const uint16_t *q_tail, *k_tail, *v_tail;
  uint16_t* o_tail;
  int Tcq, Tck, Tfull;
  float *lse_out, *rs_out, *rr_out;
  const uint16_t* states;  // [B,Hkv,nstf,128 (value d),128 (feature f)] bf16: S^T at key position base+128*i
  int B, T, Hq, Hkv, G, W, gap, nstf, ntile;  // W: window rounded up to 64; true window = W - gap
  int qt0;  // first query tile that is computed; q, o and the saved tensors hold rows 128 qt0 .. T-1 only
  float scale_log2, eps;
  float inv_d;  // 1 / head size the RMS norms average over (1/64 when the rows are zero-padded from 64 to 128)
};

// One 32-key sub-tile of the softmax branch for this wave's 32 queries (lane = query):
// S^T = K Q^T, running-max update, P^T = 2^(c S^T - m), O^T += V^T P^T.
// `m` is the reference maximum in scaled log2 units.  It is only raised (and O, l rescaled) when some
// row's maximum exceeds it by more than RESCALE_TH, so P stays below 2^RESCALE_TH and almost every
// sub-tile takes the short path: 16 fma, 8 max3, 16 exp, 16 add, 8 cvt per lane.  The exponent
// arguments x = c*s - m are formed first and the maximum is taken over them (they are already needed,
// and being fma results they need no NaN quieting).  `masked` is wave-uniform: only the window-edge and
// diagonal sub-tiles pay for the per-element mask.  CUR (LDS buffer) and KS (sub-tile) are compile-time
// so every LDS address is a per-lane register plus an immediate.
constexpr float RESCALE_TH = 8.f;
constexpr float M_INIT = -1.0e30f;  // finite "minus infinity" for the running maximum

// The sweep is software-pipelined per wave over its sequence of 32-key sub-tiles j (upper keys first):
// step j issues, in one instruction stream, the S^T chain of sub-tile j+1 (matrix cores), the softmax of
// sub-tile j (vector ALU) and the O^T update of sub-tile j-1 (matrix cores), so the two kinds of work
// overlap inside every wave instead of relying on another wave being in the opposite phase.

// A: S^T = K Q^T for sub-tile KS of the K tile in buffer KB
template <int KB, int KS>
__device__ __forceinline__ void qk_chain(const unsigned char* smem, const LaneOff& lo, const bf16x8_t (&qop)[8],
                                         f32x16_t& s) {
  const unsigned char* kt = smem + KB * 16384;
  s = f32x16_t{0};
#pragma unroll
  for (int dk = 0; dk < 8; ++dk) s = mfma32(lds_row(kt, lo, 32 * KS, dk), qop[dk], s);
}

// C: O^T += V^T P^T for sub-tile KS of the V tile in buffer VB
template <int VB, int KS>
__device__ __forceinline__ void pv_chain(const unsigned char* smem, const LaneOff& lo, const bf16x8_t (&pop)[2],
                                         f32x16_t (&oacc)[4]) {
  const unsigned char* vt = smem + 32768 + VB * 16384;
#pragma unroll
  for (int mf = 0; mf < 2; ++mf)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = mfma32(lds_trp(vt, lo, 32 * KS + 16 * mf, dt), pop[mf], oacc[dt]);
}

struct SweepGeom {
  int kt_lo, ntiles, qa, W;
  // first key of sub-tile j (tile j/2 counted from the diagonal, upper half first)
  __device__ __forceinline__ int ka(int j) const { return kt_lo + 64 * (ntiles - 1 - (j >> 1)) + 32 * (1 - (j & 1)); }
  // every (query, key) pair of the wave's 32 queries and the sub-tile's 32 keys is inside the window
  __device__ __forceinline__ bool full(int j) const {
    const int k = ka(j);
    return k + 31 <= qa && k >= qa + 31 - W + 1;
  }
};

// Step j with R = j % 4 (fixes which LDS buffers / halves sub-tiles j+1 and j-1 live in).  Every wave runs
// every step of the work-group's key range: sub-tiles outside a wave's own window are fully masked (their
// probabilities are exactly 0), which costs a few percent of the matrix work and keeps one straight
// code path.  Two scheduling regions, each pairing a matrix-core chain with vector work:
//   1. S^T(j+1) = K Q^T          ||  exponent arguments x = c*S^T(j) - m and their row maximum
//   2. O^T += V^T P^T(j-1)       ||  P^T(j) = 2^x, row sums, bf16 packing
// The reference maximum m is raised only when some row exceeds it by RESCALE_TH (rare); the rescale of
// O is applied after region 2, i.e. after the update that was still expressed against the old m.
template <int R, bool DO_C>
__device__ __forceinline__ void sweep_step(const unsigned char* smem, const LaneOff& lo, const SweepGeom& gm, int j,
                                           int myq, float scale_log2, const bf16x8_t (&qop)[8], f32x16_t (&oacc)[4],
                                           float& m, float& l, f32x16_t& s_cur, bf16x8_t (&p_prev)[2], bool& pend,
                                           float& alpha_pend, int lane) {
  constexpr int KS = R & 1;                           // sub-tile half of both j+1 and j-1
  constexpr int KB = (R == 1 || R == 2) ? 1 : 0;      // K buffer of sub-tile j+1
  constexpr int VB = (R == 0 || R == 3) ? 1 : 0;      // V buffer of sub-tile j-1
  const int h = lane >> 5;
  if (pend) {  // the rescale of O the previous step left behind (rare; wave-uniform)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] *= alpha_pend;
    pend = false;
  }
  if (!gm.full(j)) {  // wave-uniform: window edge, diagonal, or a sub-tile this wave does not see at all
    const int ka = gm.ka(j);
    // in the window <=> 0 <= query - key < W: one unsigned compare per element against a per-lane base
    const unsigned dist0 = (unsigned)(myq - ka - 4 * h);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      s_cur[i] = (dist0 - (unsigned)(8 * (i >> 2) + (i & 3)) < (unsigned)gm.W) ? s_cur[i] : -INFINITY;
  }
  // ---- region 1
  f32x16_t s_next;
  qk_chain<KB, KS>(smem, lo, qop, s_next);
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = __builtin_fmaf(s_cur[i], scale_log2, -m);
  float mx = fmaxf(fmaxf(x[0], x[1]), x[2]);
#pragma unroll
  for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, x[i]), x[i + 1]);
  mx = half_max(fmaxf(mx, x[15]));
  __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // 3 VALU
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 LDS read
  }
  const bool trig = __builtin_amdgcn_ballot_w64(mx > RESCALE_TH) != 0;
  if (trig) {
    float sm = fmaxf(s_cur[0], s_cur[1]);
#pragma unroll
    for (int i = 2; i < 16; ++i) sm = fmaxf(sm, s_cur[i]);
    const float m_new = fmaxf(m, half_max(sm) * scale_log2);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    l *= alpha;
    // O is rescaled at the start of the next step: this step's O update below is still expressed against the
    // old m, and keeping the rescale out of this place leaves the update and the exponentials in one block
    // of straight-line code, where they overlap
    pend = true;
    alpha_pend = alpha;
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = __builtin_fmaf(s_cur[i], scale_log2, -m);
  }
  // ---- region 2
  if (DO_C) pv_chain<VB, KS>(smem, lo, p_prev, oacc);
  float ps = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) { x[i] = fast_exp2(x[i]); ps += x[i]; }
  l += ps;
  p_prev[0] = pack_bf16x8(&x[0]);
  p_prev[1] = pack_bf16x8(&x[8]);
  if (DO_C) {
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // 6 VALU
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // 2 LDS reads
    }
  }
  s_cur = s_next;
}

// GAP: the window is not a multiple of 64 (a.gap > 0); the aligned case compiles without the extra key tile.
// FM: feature map of the linear branch (FM_* in mfma.hpp).
template <bool GAP, int FM>
__global__ __launch_bounds__(256, 2) void fwd_fused_kernel(FastFwdArgs a) {
  __shared__ __align__(16) unsigned char smem[65536];
  const int lane = lane_id(), w = wave_id();
  const int r32 = lane & 31, h = lane >> 5;
  const LaneOff lo = make_lane_off(lane);
  const int W = a.W, Hq = a.Hq, Hkv = a.Hkv, G = a.G;

  // work id: consecutive ids share a KV head (its G query heads, then the next query tile); each XCD
  // (blockIdx % 8) gets one contiguous range of ids so K/V tiles are reused out of its own L2
  const int total = gridDim.x;
  const int bid = blockIdx.x;
  int wid = (total % 8 == 0) ? (bid % 8) * (total / 8) + bid / 8 : bid;
  const int hh = wid % G; wid /= G;
  const int ntq = a.ntile - a.qt0, Tq = 128 * ntq;  // query tiles and query rows per sequence
  const int qt = a.ntile - 1 - wid % ntq; wid /= ntq;  // late tiles first: they see the most keys (causal / start-up tiles)
  const int g = wid % Hkv;
  const int b = wid / Hkv;
  const int hq = g * G + hh;
  const int t0 = qt * 128;
  const size_t qstride = (size_t)Hq * 128, kstride = (size_t)Hkv * 128;
  const size_t qtile_off = ((size_t)(b * Tq + t0 - 128 * a.qt0) * Hq + hq) * 128;  // in the saved tensors
  const uint16_t* q_tile = split_rows(a.q, a.q_tail, b, t0 - 128 * a.qt0, a.Tcq, a.Tfull, Hq, hq);
  uint16_t* o_tile = split_rows(a.o, a.o_tail, b, t0 - 128 * a.qt0, a.Tcq, a.Tfull, Hq, hq);
  // first row of a 64-key tile of this KV head
  auto k_rows = [&](int row) { return split_rows(a.k, a.k_tail, b, row, a.Tck, a.Tfull, Hkv, g); };
  auto v_rows = [&](int row) { return split_rows(a.v, a.v_tail, b, row, a.Tck, a.Tfull, Hkv, g); };
  const int myq = t0 + 32 * w + r32;
  const size_t stat_off = (size_t)(b * Hq + hq) * Tq + myq - 128 * a.qt0;

  // ------------------------------------------------------------------ softmax branch
  // key tiles of 64 from the diagonal (n = 0) down to kt_lo (n = ntiles-1); tile n uses LDS buffer n & 1.
  // K runs one tile ahead of V through the buffers (the S^T chain of a sub-tile is issued one step early).
  const int kt_lo = max(0, t0 - W);
  const int ntiles = (t0 + 128 - kt_lo) / 64;  // >= 2
  const DmaLane dl = make_dma_lane(lane, kstride);
  auto load_k = [&](int n) {
    tile_load_async_s<4>(k_rows(kt_lo + 64 * (ntiles - 1 - n)), kstride, smem + (n & 1) * 16384, w * 4, dl);
  };
  auto load_v = [&](int n) {
    tile_load_async_s<4>(v_rows(kt_lo + 64 * (ntiles - 1 - n)), kstride, smem + 32768 + (n & 1) * 16384, w * 4, dl);
  };
  load_k(0);
  load_v(0);
  load_k(1);
  bf16x8_t qop[8];
  {
    const uint16_t* qp = q_tile + (size_t)(32 * w + r32) * qstride + 8 * h;
#pragma unroll
    for (int dk = 0; dk < 8; ++dk) qop[dk] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * dk);
  }
  wait_vmem();
  __syncthreads();
  f32x16_t oacc[4] = {{0}, {0}, {0}, {0}};
  float m = M_INIT, l = 0.f;
  SweepGeom gm;
  gm.kt_lo = kt_lo; gm.ntiles = ntiles; gm.qa = t0 + 32 * w; gm.W = W - (GAP ? a.gap : 0);
  f32x16_t s_cur;
  bf16x8_t p_prev[2];
  bool pend = false;
  float alpha_pend = 1.f;
  qk_chain<0, 1>(smem, lo, qop, s_cur);
  // step 0 has no earlier sub-tile to fold in; the step after the last one only folds
  sweep_step<0, false>(smem, lo, gm, 0, myq, a.scale_log2, qop, oacc, m, l, s_cur, p_prev, pend, alpha_pend, lane);
  for (int n = 0; n < ntiles; n += 2) {
    if (n > 0) sweep_step<0, true>(smem, lo, gm, 2 * n, myq, a.scale_log2, qop, oacc, m, l, s_cur, p_prev, pend, alpha_pend, lane);
    wait_vmem();
    __syncthreads();
    if (n + 2 < ntiles) load_k(n + 2);
    if (n + 1 < ntiles) load_v(n + 1);
    sweep_step<1, true>(smem, lo, gm, 2 * n + 1, myq, a.scale_log2, qop, oacc, m, l, s_cur, p_prev, pend, alpha_pend, lane);
    if (n + 1 < ntiles) {
      sweep_step<2, true>(smem, lo, gm, 2 * n + 2, myq, a.scale_log2, qop, oacc, m, l, s_cur, p_prev, pend, alpha_pend, lane);
      wait_vmem();
      __syncthreads();
      if (n + 3 < ntiles) load_k(n + 3);
      if (n + 2 < ntiles) load_v(n + 2);
      sweep_step<3, true>(smem, lo, gm, 2 * n + 3, myq, a.scale_log2, qop, oacc, m, l, s_cur, p_prev, pend, alpha_pend, lane);
    }
  }
  if (pend) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] *= alpha_pend;
  }
  if (ntiles & 1) pv_chain<0, 0>(smem, lo, p_prev, oacc);
  else pv_chain<1, 0>(smem, lo, p_prev, oacc);
  __syncthreads();
  // the two lowest key tiles are still resident: tile `it` sits in buffer (ntiles-1-it) & 1

  l = half_sum(l);
  const float inv_l = 1.f / l;
  float ss = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    oacc[dt] *= inv_l;
#pragma unroll
    for (int i = 0; i < 16; ++i) ss += oacc[dt][i] * oacc[dt][i];
  }
  ss = half_sum(ss);
  const float rs_val = rsqrtf(ss * a.inv_d + a.eps);
  // key tile of the intra-chunk part starts at j0 = t0 - W; when W % 128 == 64 the first query tile that
  // reaches past the window has j0 = -64: no state yet (S = 0) and only its upper 64 keys exist
  // (with gap > 0 the tile at j0 = -128 reaches keys too: only through the extra 64 keys fetched below)
  const int j0 = t0 - W;
  const bool has_lin = j0 > -128 || (GAP && j0 == -128);
  if (a.xs_out) {
    if (!has_lin) {   // (with a linear branch LDS still holds the tiles that branch works on: x_s is stored after it)
      float vals[4][16];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) vals[dt][i] = oacc[dt][i];
      store_tile_transposed(smem, vals, a.xs_out + qtile_off, qstride, w, lane);
    }
  }
  // x_s * r_s stays in fp32 across the linear branch: the output is rounded once, after the sum of the branches
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) oacc[dt] *= rs_val;
  const float lse_val = (m + log2f(l)) * LN2;

  // ------------------------------------------------------------------ linear branch
  // intra-chunk part on the resident tiles (phi applied to K in place), then the state product
  f32x16_t xr[4] = {{0}, {0}, {0}, {0}};
  float rr_val = rsqrtf(a.eps);
  if (has_lin) {
    const bool has_state = j0 >= 0;
    const int shift = has_state ? 0 : 1;                  // chunk tile ti is softmax tile ti - shift
    const int buf0 = (ntiles - 1 + shift) & 1;            // buffer of chunk tile 0 (tile 1 is the other one)
    bf16x8_t qfop[8];
    {
      float x[64];
#pragma unroll
      for (int dk = 0; dk < 8; ++dk) unpack_bf16x8(qop[dk], &x[8 * dk]);
      phi_rows<FM>(x, qfop);
    }
    const bool has_res = j0 > -128;  // the resident tiles hold keys of this chunk
    if (has_res) phi_tiles_inplace<FM>(has_state ? smem + buf0 * 16384 : nullptr, smem + (buf0 ^ 1) * 16384);
    __syncthreads();
    // Key sub-tile u (keys j0 + 32u .. +31) meets query block w when 32u <= 32w + 31 + gap; a query sees
    // key_local <= q_local + gap.  Sub-tiles 0..3 are resident; with gap > 0 the top queries also reach
    // into the next 64 keys, fetched afterwards.
    const int gap = GAP ? a.gap : 0;
    const int u_hi = w + ((31 + gap) >> 5);
    auto intra_unit = [&](const unsigned char* kt, const unsigned char* vt, int ks, int u) {
      f32x16_t c = {0};
#pragma unroll
      for (int dk = 0; dk < 8; ++dk) c = mfma32(lds_row(kt, lo, 32 * ks, dk), qfop[dk], c);
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
        for (int dt = 0; dt < 4; ++dt) xr[dt] = mfma32(lds_trp(vt, lo, 32 * ks + 16 * mf, dt), cop[mf], xr[dt]);
      }
    };
    for (int u = has_state ? 0 : (has_res ? 2 : 4); u <= min(3, u_hi); ++u) {
      const int bsel = buf0 ^ (u >> 1);
      intra_unit(smem + bsel * 16384, smem + 32768 + bsel * 16384, u & 1, u);
    }
    __syncthreads();
    if (GAP) {
      tile_load_async<4>(k_rows(j0 + 128), kstride, smem, w * 4, lane);
      tile_load_async<4>(v_rows(j0 + 128), kstride, smem + 32768, w * 4, lane);
      wait_vmem();
      __syncthreads();
      phi_tiles_inplace<FM>(smem, nullptr);
      __syncthreads();
      for (int u = 4; u <= min(5, u_hi); ++u) intra_unit(smem, smem + 32768, u & 1, u);
      __syncthreads();
    }
    if (has_state) {
      const uint16_t* sbase = a.states + ((size_t)(b * Hkv + g) * a.nstf + j0 / 128) * 16384;
      tile_load_async<8>(sbase, 128, smem, w * 8, lane);
      wait_vmem();
      __syncthreads();
#pragma unroll
      for (int kf = 0; kf < 8; ++kf)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) xr[dt] = mfma32(lds_row(smem, lo, 32 * dt, kf), qfop[kf], xr[dt]);
      __syncthreads();
    }
    float sr = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) sr += xr[dt][i] * xr[dt][i];
    sr = half_sum(sr);
    rr_val = rsqrtf(sr * a.inv_d + a.eps);
  }
  if (a.xs_out) {
    float vals[4][16];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) vals[dt][i] = xr[dt][i];
    // (a tile without residual keys has x_r = 0, which backward knows from the tile's position: not stored)
    if (has_lin) {
      store_tile_transposed(smem, vals, a.xr_out + qtile_off, qstride, w, lane);
      // x_s = (x_s r_s) / r_s: the accumulators hold the normalised rows by now
      const float inv_rs = 1.f / rs_val;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) vals[dt][i] = oacc[dt][i] * inv_rs;
      store_tile_transposed(smem, vals, a.xs_out + qtile_off, qstride, w, lane);
    }
    if (h == 0) {
      a.lse_out[stat_off] = lse_val;
      a.rs_out[stat_off] = rs_val;
      a.rr_out[stat_off] = rr_val;
    }
  }

  // ------------------------------------------------------------------ combination
  {
    float vals[4][16];
    if (!a.gs && !a.gr) {  // no gains: one multiply-add per element, no loads
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) vals[dt][i] = __builtin_fmaf(rr_val, xr[dt][i], oacc[dt][i]);
    } else {
      // the head's two gain rows go through LDS (free since the last barrier; the store below uses [0, 32K))
      float* gl = reinterpret_cast<float*>(smem + 32768);
      if (threadIdx.x < 128) {
        gl[threadIdx.x] = a.gs ? a.gs[hq * 128 + threadIdx.x] : 1.f;
        gl[128 + threadIdx.x] = a.gr ? a.gr[hq * 128 + threadIdx.x] : 1.f;
      }
      __syncthreads();
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const int d0 = 32 * dt + 8 * i4 + 4 * h;
          const float4 g1 = *reinterpret_cast<const float4*>(gl + d0);
          const float4 g2 = *reinterpret_cast<const float4*>(gl + 128 + d0);
          const float ga[4] = {g1.x, g1.y, g1.z, g1.w}, gb[4] = {g2.x * rr_val, g2.y * rr_val, g2.z * rr_val, g2.w * rr_val};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * i4 + e;
            vals[dt][i] = ga[e] * oacc[dt][i] + gb[e] * xr[dt][i];
          }
        }
    }
    store_tile_transposed(smem, vals, o_tile, qstride, w, lane);
  }
}

}  // namespace

void fast_fwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs, const float* gr,
              void* o, const SavedPtrs& sv, float* U, void* states, hipStream_t st, int qt0, const float* state0,
              const RaggedTails* tails) {
  const FastFwdPlan pl = fast_fwd_plan(dm);
  // `states` receives every chunk state; with a state stride the stored subset also goes to `saved`
  if (pl.nstf > 0)
    rla_forward_states(dm, pl, k, v, U, states, st, state0, tails, sv.state_stride > 1 ? sv.states : nullptr, nullptr,
                       sv.state_stride);
  FastFwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.gs = gs; a.gr = gr;
  a.o = (uint16_t*)o; a.xs_out = (uint16_t*)sv.xs; a.xr_out = (uint16_t*)sv.xr;
  a.lse_out = sv.lse; a.rs_out = sv.rs; a.rr_out = sv.rr;
  a.states = (const uint16_t*)states;
  a.B = dm.B; a.T = dm.T; a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.G = dm.G; a.W = pl.W; a.gap = pl.gap; a.nstf = pl.nstf;
  a.ntile = dm.T / 128; a.qt0 = qt0;
  // the caller's tensors: q and o hold the computed tiles only; with tails (always qt0 == 0) Tc rows per sequence
  a.q_tail = tails ? (const uint16_t*)tails->q : nullptr; a.k_tail = tails ? (const uint16_t*)tails->k : nullptr;
  a.v_tail = tails ? (const uint16_t*)tails->v : nullptr; a.o_tail = tails ? (uint16_t*)tails->o : nullptr;
  a.Tcq = tails ? tails->Tc : dm.T - 128 * qt0;
  a.Tck = tails ? tails->Tc : dm.T;
  a.Tfull = tails ? tails->Tc / 128 * 128 : INT_MAX;
  a.scale_log2 = dm.scale * LOG2E; a.eps = dm.eps;
  ProfScope ps("fwd_fused_kernel", st);
  const dim3 grid((a.ntile - qt0) * dm.Hq * dm.B);
  a.inv_d = 1.f / (float)dm.Dv;
#define RATTN_FWD_LAUNCH(FM_)                                             \
  do {                                                                    \
    if (a.gap > 0) fwd_fused_kernel<true, FM_><<<grid, 256, 0, st>>>(a);  \
    else fwd_fused_kernel<false, FM_><<<grid, 256, 0, st>>>(a);           \
  } while (0)
  switch (feature_map_variant(dm)) {
    case FM_RELU: RATTN_FWD_LAUNCH(FM_RELU); break;
    case FM_IDENTITY: RATTN_FWD_LAUNCH(FM_IDENTITY); break;
    case FM_SOFTMAX64: RATTN_FWD_LAUNCH(FM_SOFTMAX64); break;
    default: RATTN_FWD_LAUNCH(FM_SOFTMAX); break;
  }
#undef RATTN_FWD_LAUNCH
}

}  // namespace rattn
