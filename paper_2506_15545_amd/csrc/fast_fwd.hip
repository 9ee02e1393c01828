// MFMA forward of the RAttention layer for bf16, D = 128, T % 128 == 0, W % 64 == 0 (or W >= T).
//
// One work-group (4 waves) owns 128 consecutive queries of one head; wave w owns 32 of them.
// Everything is computed TRANSPOSED so that a lane always owns one query (column) of the MFMA
// results and all row statistics are lane-local (plus one exchange with lane^32):
//   softmax branch (Sec. 2.1):  S^T = K Q^T  ->  online softmax  ->  O^T += V^T P^T
//   linear branch (Eqs. 2-4) :  X^T = St Qf^T  +  V^T (M^T .* (Kf Qf^T)),  St = S_[j]^T (bf16, from the
//                               state pre-pass), Qf/Kf = phi(Q)/phi(K) computed on the operand registers
//   combination (Sec. 3.2)   :  o = gs * x_s * r_s + gr * x_r * r_r, transposed through LDS for
//                               coalesced stores
// K/V tiles (64 keys) stream through a double buffer in LDS with direct-to-LDS loads; the linear
// branch runs first (its normalised result is carried as packed bf16), then the softmax branch walks
// its key tiles from the diagonal downwards, so every row's running maximum is finite from the start.
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"

namespace rattn {

namespace {

struct FastFwdArgs {
  const uint16_t *q, *k, *v;
  const float *gs, *gr;
  uint16_t *o, *xs_out, *xr_out;
  float *lse_out, *rs_out, *rr_out;
  const uint16_t* states;  // [B,Hkv,nstf,128 (value d),128 (feature f)] bf16: S^T at key position base+128*i
  int B, T, Hq, Hkv, G, W, nstf, ntile;
  float scale_log2, eps;
};

// One 32-key sub-tile of the softmax branch for this wave's 32 queries (lane = query):
// S^T = K Q^T, running-max update, P^T = 2^(c S^T - m), O^T += V^T P^T.
// `m` is the reference maximum in scaled log2 units.  It is only raised (and O, l rescaled) when some
// row's maximum exceeds it by more than RESCALE_TH, so P stays below 2^RESCALE_TH and most sub-tiles skip
// the 64-register rescale.  `masked` is wave-uniform: only the window-edge and diagonal sub-tiles pay
// for the per-element mask.
constexpr float RESCALE_TH = 8.f;

__device__ __forceinline__ void swa_subtile(const unsigned char* kt, const unsigned char* vt, int ks, int ka, int myq,
                                            int W, bool masked, float scale_log2, const bf16x8_t (&qop)[8],
                                            f32x16_t (&oacc)[4], float& m, float& l, int lane, const LaneOff& lo) {
  const int h = lane >> 5;
  f32x16_t s = {0};
#pragma unroll
  for (int dk = 0; dk < 8; ++dk) s = mfma32(lds_row(kt, lo, 32 * ks, dk), qop[dk], s);
  if (masked) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = ka + 8 * (i >> 2) + 4 * h + (i & 3);
      const bool ok = key <= myq && key > myq - W;
      s[i] = ok ? s[i] : -INFINITY;
    }
  }
  float mx = fmaxf(s[0], s[1]);
#pragma unroll
  for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(s[i], s[i + 1]));
  mx = half_max(mx) * scale_log2;
  if (__builtin_amdgcn_ballot_w64(mx - m > RESCALE_TH) != 0) {
    const float m_new = fmaxf(m, mx);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] *= alpha;
  }
  float x[16], ps = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) { x[i] = fast_exp2(__builtin_fmaf(s[i], scale_log2, -m)); ps += x[i]; }
  l += ps;
  bf16x8_t pop[2] = {pack_bf16x8(&x[0]), pack_bf16x8(&x[8])};
#pragma unroll
  for (int mf = 0; mf < 2; ++mf) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = mfma32(lds_trp(vt, lo, 32 * ks + 16 * mf, dt), pop[mf], oacc[dt]);
  }
}

__global__ __launch_bounds__(256, 2) void fwd_fused_kernel(FastFwdArgs a) {
  __shared__ __align__(16) unsigned char smem[65536];
  const int lane = lane_id(), w = wave_id();
  const int r32 = lane & 31, h = lane >> 5;
  const LaneOff lo = make_lane_off(lane);
  const int T = a.T, W = a.W, Hq = a.Hq, Hkv = a.Hkv, G = a.G;

  // work id: consecutive ids share a KV head (its G query heads, then the next query tile); each XCD
  // (blockIdx % 8) gets one contiguous range of ids so K/V tiles are reused out of its own L2
  const int total = gridDim.x;
  const int bid = blockIdx.x;
  int wid = (total % 8 == 0) ? (bid % 8) * (total / 8) + bid / 8 : bid;
  const int hh = wid % G; wid /= G;
  const int qt = wid % a.ntile; wid /= a.ntile;
  const int g = wid % Hkv;
  const int b = wid / Hkv;
  const int hq = g * G + hh;
  const int t0 = qt * 128;
  const size_t qstride = (size_t)Hq * 128, kstride = (size_t)Hkv * 128;
  const size_t qtile_off = ((size_t)(b * T + t0) * Hq + hq) * 128;
  const uint16_t* kbase = a.k + ((size_t)b * T * Hkv + g) * 128;
  const uint16_t* vbase = a.v + ((size_t)b * T * Hkv + g) * 128;
  const int myq = t0 + 32 * w + r32;
  const size_t stat_off = (size_t)(b * Hq + hq) * T + myq;

  bf16x8_t qop[8];
  {
    const uint16_t* qp = a.q + qtile_off + (size_t)(32 * w + r32) * qstride + 8 * h;
#pragma unroll
    for (int dk = 0; dk < 8; ++dk) qop[dk] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * dk);
  }

  // ------------------------------------------------------------------ linear branch
  bf16x2_t yr[4][8];  // x_r * r_r, packed
  float rr_val = rsqrtf(a.eps);
  // key tile of the intra-chunk part starts at j0 = t0 - W; when W % 128 == 64 the first query tile that
  // reaches past the window has j0 = -64: no state yet (S = 0) and only its upper 64 keys exist
  const int j0 = t0 - W;
  if (j0 > -128) {
    const bool has_state = j0 >= 0;
    bf16x8_t qfop[8];
    {
      float x[64];
#pragma unroll
      for (int dk = 0; dk < 8; ++dk) unpack_bf16x8(qop[dk], &x[8 * dk]);
      phi_rows(x, qfop);
    }
    f32x16_t xr[4] = {{0}, {0}, {0}, {0}};
    if (has_state) {
      const uint16_t* sbase = a.states + ((size_t)(b * Hkv + g) * a.nstf + j0 / 128) * 16384;
      tile_load_async<8>(sbase, 128, smem, w * 8, lane);
      tile_load_async<4>(vbase + (size_t)j0 * kstride, kstride, smem + 32768, w * 4, lane);
    }
    tile_load_async<4>(vbase + (size_t)(j0 + 64) * kstride, kstride, smem + 49152, w * 4, lane);
    wait_vmem();
    __syncthreads();
    if (has_state) {
#pragma unroll
      for (int kf = 0; kf < 8; ++kf)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
          xr[dt] = mfma32(lds_row(smem, lo, 32 * dt, kf), qfop[kf], xr[dt]);
    }
    __syncthreads();
    if (has_state) tile_load_async<4>(kbase + (size_t)j0 * kstride, kstride, smem, w * 4, lane);
    tile_load_async<4>(kbase + (size_t)(j0 + 64) * kstride, kstride, smem + 16384, w * 4, lane);
    wait_vmem();
    __syncthreads();
    if (has_state) phi_tile_inplace(smem, 128);
    else phi_tile_inplace(smem + 16384, 64);
    __syncthreads();
    for (int u = has_state ? 0 : 2; u <= w; ++u) {
      const unsigned char* kt = smem + (u >> 1) * 16384;
      const unsigned char* vt = smem + 32768 + (u >> 1) * 16384;
      const int ks = u & 1;
      f32x16_t c = {0};
#pragma unroll
      for (int dk = 0; dk < 8; ++dk) c = mfma32(lds_row(kt, lo, 32 * ks, dk), qfop[dk], c);
      float cv[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key_local = 32 * u + 8 * (i >> 2) + 4 * h + (i & 3);
        cv[i] = (u == w && key_local > 32 * w + r32) ? 0.f : c[i];
      }
      bf16x8_t cop[2] = {pack_bf16x8(&cv[0]), pack_bf16x8(&cv[8])};
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
    #pragma unroll
        for (int dt = 0; dt < 4; ++dt) xr[dt] = mfma32(lds_trp(vt, lo, 32 * ks + 16 * mf, dt), cop[mf], xr[dt]);
      }
    }
    __syncthreads();
    float ss = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) ss += xr[dt][i] * xr[dt][i];
    ss = half_sum(ss);
    rr_val = rsqrtf(ss * (1.f / 128.f) + a.eps);
    if (a.xr_out) {
      float vals[4][16];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) vals[dt][i] = xr[dt][i];
      store_tile_transposed(smem, vals, a.xr_out + qtile_off, qstride, w, lane);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        f32x2_t f = {xr[dt][2 * i] * rr_val, xr[dt][2 * i + 1] * rr_val};
        yr[dt][i] = __builtin_convertvector(f, bf16x2_t);
      }
  } else {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        f32x2_t f = {0.f, 0.f};
        yr[dt][i] = __builtin_convertvector(f, bf16x2_t);
      }
    if (a.xr_out) {
      const int tid = threadIdx.x;
      const uint4 z = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int id = tid + 256 * i;
        *reinterpret_cast<uint4*>(a.xr_out + qtile_off + (size_t)(id >> 4) * qstride + (id & 15) * 8) = z;
      }
    }
  }

  // ------------------------------------------------------------------ softmax branch
  f32x16_t oacc[4] = {{0}, {0}, {0}, {0}};
  float m = -INFINITY, l = 0.f;
  const int kt_lo = max(0, t0 - W);
  const int ntiles = (t0 + 128 - kt_lo) / 64;
  {
    const int kt0 = kt_lo + 64 * (ntiles - 1);
    tile_load_async<4>(kbase + (size_t)kt0 * kstride, kstride, smem, w * 4, lane);
    tile_load_async<4>(vbase + (size_t)kt0 * kstride, kstride, smem + 32768, w * 4, lane);
    wait_vmem();
    __syncthreads();
  }
  const int qa = t0 + 32 * w, qb = qa + 31;
  for (int n = 0; n < ntiles; ++n) {
    const int it = ntiles - 1 - n;
    const int cur = n & 1;
    if (n + 1 < ntiles) {
      const int ktn = kt_lo + 64 * (it - 1);
      tile_load_async<4>(kbase + (size_t)ktn * kstride, kstride, smem + (cur ^ 1) * 16384, w * 4, lane);
      tile_load_async<4>(vbase + (size_t)ktn * kstride, kstride, smem + 32768 + (cur ^ 1) * 16384, w * 4, lane);
    }
    const unsigned char* kt = smem + cur * 16384;
    const unsigned char* vt = smem + 32768 + cur * 16384;
    const int kt0 = kt_lo + 64 * it;
#pragma unroll
    for (int ks = 1; ks >= 0; --ks) {
      const int ka = kt0 + 32 * ks;
      const bool need = ka <= qb && ka + 31 >= qa - W + 1;
      if (need) {
        const bool full = ka + 31 <= qa && ka >= qb - W + 1;
        swa_subtile(kt, vt, ks, ka, myq, W, !full, a.scale_log2, qop, oacc, m, l, lane, lo);
      }
    }
    wait_vmem();
    __syncthreads();
  }

  // ------------------------------------------------------------------ combination
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
  const float rs_val = rsqrtf(ss * (1.f / 128.f) + a.eps);
  if (a.xs_out) {
    float vals[4][16];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) vals[dt][i] = oacc[dt][i];
    store_tile_transposed(smem, vals, a.xs_out + qtile_off, qstride, w, lane);
    if (h == 0) {
      a.lse_out[stat_off] = (m + log2f(l)) * LN2;
      a.rs_out[stat_off] = rs_val;
      a.rr_out[stat_off] = rr_val;
    }
  }
  {
    float vals[4][16];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d0 = 32 * dt + 8 * i4 + 4 * h;
        float4 g1 = make_float4(1.f, 1.f, 1.f, 1.f), g2 = g1;
        if (a.gs) g1 = *reinterpret_cast<const float4*>(a.gs + hq * 128 + d0);
        if (a.gr) g2 = *reinterpret_cast<const float4*>(a.gr + hq * 128 + d0);
        const float ga[4] = {g1.x, g1.y, g1.z, g1.w}, gb[4] = {g2.x, g2.y, g2.z, g2.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * i4 + e;
          const float y = (float)yr[dt][i >> 1][i & 1];
          vals[dt][i] = ga[e] * oacc[dt][i] * rs_val + gb[e] * y;
        }
      }
    store_tile_transposed(smem, vals, a.o + qtile_off, qstride, w, lane);
  }
}

}  // namespace

bool fast_fwd_supported(const LayerDims& dm, int dtype) {
  if (dtype != 1 || dm.D != 128 || dm.T % 128 != 0) return false;
  if (!(dm.scale > 0.f)) return false;
  if (dm.W < dm.T && dm.W % 64 != 0) return false;
  return true;
}

FastFwdPlan fast_fwd_plan(const LayerDims& dm) {
  FastFwdPlan p;
  p.W = dm.W >= dm.T ? dm.T : dm.W;
  p.base = p.W % 128;
  p.nstf = dm.T / 128 - (p.W + 127) / 128;
  if (p.nstf < 0) p.nstf = 0;
  p.nchunks = p.nstf > 0 ? (p.nstf - 1) + (p.base > 0 ? 1 : 0) : 0;
  p.u_bytes = (size_t)dm.B * dm.Hkv * p.nchunks * 16384 * 4;
  p.state_bytes = (size_t)dm.B * dm.Hkv * p.nstf * 16384 * 2;
  return p;
}

void fast_fwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs, const float* gr,
              void* o, const SavedPtrs& sv, float* U, void* states, hipStream_t st) {
  const FastFwdPlan pl = fast_fwd_plan(dm);
  if (pl.nstf > 0) rla_forward_states(dm, pl, k, v, U, states, st);
  FastFwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.gs = gs; a.gr = gr;
  a.o = (uint16_t*)o; a.xs_out = (uint16_t*)sv.xs; a.xr_out = (uint16_t*)sv.xr;
  a.lse_out = sv.lse; a.rs_out = sv.rs; a.rr_out = sv.rr;
  a.states = (const uint16_t*)states;
  a.B = dm.B; a.T = dm.T; a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.G = dm.G; a.W = pl.W; a.nstf = pl.nstf;
  a.ntile = dm.T / 128;
  a.scale_log2 = dm.scale * LOG2E; a.eps = dm.eps;
  ProfScope ps("fwd_fused_kernel", st);
  fwd_fused_kernel<<<dim3(a.ntile * dm.Hq * dm.B), 256, 0, st>>>(a);
}

}  // namespace rattn
