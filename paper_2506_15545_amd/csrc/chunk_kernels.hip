// Chunked prefill: the layer's forward for the next Tc tokens of sequences whose first pos0 tokens are only
// present as what the decode path keeps (Sec. 2.1: a ring of the last W keys/values; Sec. 2.2 / Eq. 4: the state
// S0 = sum over s < pos0 - W of phi(k_s)^T v_s).
//
// The sequence that the forward kernels see is [ring tokens in time order ; the new chunk]: every new query then
// finds its whole window, and every key that has left some query's window but is still in the ring, in the
// tensor.  What the tensor does not hold is the contribution of the keys before the ring; the linear branch is
// linear in its state, so it is added afterwards:  x_r = x_r(local) + phi(q) S0, after which the second RMS and
// the branch sum (Sec. 3.2) are redone for the new rows from the pre-norm values the forward saved.
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"

namespace rattn {

namespace {

// Rows j < R of the concatenated tensors come from the rings (token pos0 - R + j sits in slot (pos0 - R + j) % W),
// rows j >= R from the chunk; the query rows in front of the chunk are zero (their outputs are not used).  With
// q = NULL only K and V are gathered.
// One thread per 16 bytes; `row_vecs` = 16-byte pieces per row of one head.
__global__ __launch_bounds__(256) void chunk_concat_kernel(const uint4* __restrict__ q, const uint4* __restrict__ k,
                                                           const uint4* __restrict__ v, const uint4* __restrict__ k_ring,
                                                           const uint4* __restrict__ v_ring, uint4* __restrict__ qc,
                                                           uint4* __restrict__ kc, uint4* __restrict__ vc, int B, int Tc,
                                                           int R, int Hq, int Hkv, int W, int pos0, int row_vecs) {
  const int L = R + Tc;
  const long long nkv = (long long)B * L * Hkv * row_vecs, nq = q ? (long long)B * L * Hq * row_vecs : 0;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < nkv + nq; i += (long long)gridDim.x * 256) {
    if (i < nkv) {
      const int c = (int)(i % row_vecs);
      long long r = i / row_vecs;
      const int g = (int)(r % Hkv); r /= Hkv;
      const int j = (int)(r % L);
      const int b = (int)(r / L);
      if (j < R) {
        const int slot = (pos0 - R + j) % W;
        const size_t src = (((size_t)b * Hkv + g) * W + slot) * row_vecs + c;
        kc[i] = k_ring[src];
        vc[i] = v_ring[src];
      } else {
        const size_t src = ((size_t)(b * Tc + j - R) * Hkv + g) * row_vecs + c;
        kc[i] = k[src];
        vc[i] = v[src];
      }
    } else {
      const long long iq = i - nkv;
      const int c = (int)(iq % row_vecs);
      long long r = iq / row_vecs;
      const int hq = (int)(r % Hq); r /= Hq;
      const int j = (int)(r % L);
      const int b = (int)(r / L);
      qc[iq] = j < R ? make_uint4(0u, 0u, 0u, 0u) : q[((size_t)(b * Tc + j - R) * Hq + hq) * row_vecs + c];
    }
  }
}

// o[b, t, :, :] = oc[b, R + t, :, :]  (state-free case: the forward's own output is final)
__global__ __launch_bounds__(256) void chunk_copy_out_kernel(const uint4* __restrict__ oc, uint4* __restrict__ o, int B,
                                                             int Tc, int R, long long row_vecs_all) {
  const long long total = (long long)B * Tc * row_vecs_all;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long c = i % row_vecs_all, r = i / row_vecs_all;
    const int t = (int)(r % Tc), b = (int)(r / Tc);
    o[i] = oc[((long long)b * (R + Tc) + R + t) * row_vecs_all + c];
  }
}

// New rows with the carried state added to the linear branch.  grid (ceil(Tc / 64), Hq, B), 256 threads: the
// work-group stages S0[b, g] (fp32 [feature][value]) in LDS, every wave takes 16 rows, a lane owns value columns
// lane and lane + 64.  Per row: phi(q) (softmax over the D features, or the ablation's ReLU / identity), x_r = x_r(saved) + phi(q) S0, second RMS
// recomputed, o = gs * x_s * r_s + gr * x_r * r_r (Sec. 3.2) with x_s, r_s as the forward saved them (in tensors of
// Ls >= R + Tc rows per sequence: the forward may have run on a zero-padded copy).
template <typename IO, typename ST, int D>
__global__ __launch_bounds__(256) void chunk_fixup_kernel(const IO* __restrict__ qc, const ST* __restrict__ xs,
                                                          const ST* __restrict__ xr, const float* __restrict__ rs,
                                                          const float* __restrict__ state, const float* __restrict__ gs,
                                                          const float* __restrict__ gr, IO* __restrict__ o, int Tc, int R,
                                                          int Ls, int Hq, int Hkv, float eps, int phi) {
  constexpr int NE = D / 64;  // elements per lane
  extern __shared__ __align__(16) float s0[];  // [D][D]
  const int hq = blockIdx.y, b = blockIdx.z, G = Hq / Hkv, g = hq / G;
  const int lane = lane_id(), w = wave_id();
  const int L = R + Tc;
  {
    const float4* src = reinterpret_cast<const float4*>(state + ((size_t)b * Hkv + g) * D * D);
    float4* dst = reinterpret_cast<float4*>(s0);
    for (int i = threadIdx.x; i < D * D / 4; i += 256) dst[i] = src[i];
  }
  __syncthreads();
  float g1[NE], g2[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) {
    g1[e] = gs ? gs[hq * D + lane + 64 * e] : 1.f;
    g2[e] = gr ? gr[hq * D + lane + 64 * e] : 1.f;
  }
  for (int i = 0; i < 16; ++i) {
    const int t = blockIdx.x * 64 + w * 16 + i;
    if (t >= Tc) break;
    const size_t roff = ((size_t)(b * L + R + t) * Hq + hq) * D;    // row of the concatenated queries
    const size_t soff = ((size_t)(b * Ls + R + t) * Hq + hq) * D;   // the same row in the saved tensors
    float x[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) x[e] = io_traits<IO>::ld(qc + roff + lane + 64 * e);
    feature_row<NE>(x, x, phi);
    float acc[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) acc[e] = io_traits<ST>::ld(xr + soff + lane + 64 * e);
#pragma unroll
    for (int fe = 0; fe < NE; ++fe) {
      for (int fl = 0; fl < 64; ++fl) {
        const float pf = bcast(x[fe], fl);
        const float* row = s0 + (size_t)(64 * fe + fl) * D;
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[e] = fmaf(pf, row[lane + 64 * e], acc[e]);
      }
    }
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < NE; ++e) ss += acc[e] * acc[e];
    const float r_r = rsqrtf(wave_sum(ss) * (1.f / D) + eps);
    const float r_s = rs[((size_t)b * Hq + hq) * Ls + R + t];
    const size_t ooff = ((size_t)(b * Tc + t) * Hq + hq) * D;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const float a = io_traits<ST>::ld(xs + soff + lane + 64 * e);
      io_traits<IO>::st(o + ooff + lane + 64 * e, g1[e] * a * r_s + g2[e] * acc[e] * r_r);
    }
  }
}

// The same for bf16, D = 128 and a concatenated length that is a multiple of 128, on the matrix cores, in the
// transposed formulation of the forward kernel (lane = query row): X^T += S0^T phi(Q)^T with S0^T rounded to bf16
// like the chunk states of the forward.  grid (tiles, Hq, B), 256 threads; tile i covers concatenated rows
// 128 (i + R / 128) .. +127, rows before the chunk (j < R) are computed and dropped.
template <int FM>
__global__ __launch_bounds__(256) void chunk_fixup_mfma_kernel(const uint16_t* __restrict__ qc, const uint16_t* __restrict__ xs,
                                                               const uint16_t* __restrict__ xr, const float* __restrict__ rs,
                                                               const float* __restrict__ state, const float* __restrict__ gs,
                                                               const float* __restrict__ gr, uint16_t* __restrict__ o, int Tc,
                                                               int R, int Hq, int Hkv, float eps) {
  __shared__ __align__(16) unsigned char smem[65536];  // [0, 32K): S0^T tile, [32K, 64K): output staging
  const int hq = blockIdx.y, b = blockIdx.z, G = Hq / Hkv, g = hq / G;
  const int lane = lane_id(), w = wave_id();
  const int r32 = lane & 31, h = lane >> 5;
  const LaneOff lo = make_lane_off(lane);
  const int L = R + Tc;
  const int j0 = 128 * (blockIdx.x + R / 128);
  {
    // S0 [f][d] fp32 -> tile row d, column f (bf16, swizzled 16-byte chunks); a thread converts 8 features of one
    // value column: coalesced global reads (consecutive d), conflict-free 16-byte LDS writes
    const float* src = state + ((size_t)b * Hkv + g) * 16384;
    for (int i = threadIdx.x; i < 2048; i += 256) {
      const int d = i & 127, c = i >> 7;
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = src[(8 * c + e) * 128 + d];
      *reinterpret_cast<bf16x8_t*>(smem + d * ROW_BYTES + ((c ^ swz(d)) << 4)) = pack_bf16x8(x);
    }
  }
  const int j = j0 + 32 * w + r32;  // this lane's row
  const size_t roff = ((size_t)(b * L + j) * Hq + hq) * 128;
  bf16x8_t qfop[8];
  {
    float x[64];
#pragma unroll
    for (int c = 0; c < 8; ++c)
      unpack_bf16x8(*reinterpret_cast<const bf16x8_t*>(qc + roff + 16 * c + 8 * h), &x[8 * c]);
    phi_rows<FM>(x, qfop);
  }
  __syncthreads();
  f32x16_t acc[4] = {{0}, {0}, {0}, {0}};
#pragma unroll
  for (int kf = 0; kf < 8; ++kf)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) acc[dt] = mfma32(lds_row(smem, lo, 32 * dt, kf), qfop[kf], acc[dt]);
  // accumulator (dt, i) = value column 32 dt + 8 (i / 4) + 4 h + i % 4 of row j
  float ss = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const bf16x4_t pv = *reinterpret_cast<const bf16x4_t*>(xr + roff + 32 * dt + 8 * i4 + 4 * h);
      const f32x4_t f = __builtin_convertvector(pv, f32x4_t);
#pragma unroll
      for (int e = 0; e < 4; ++e) { acc[dt][4 * i4 + e] += f[e]; ss += acc[dt][4 * i4 + e] * acc[dt][4 * i4 + e]; }
    }
  const float r_r = rsqrtf(half_sum(ss) * (1.f / 128.f) + eps);
  const float r_s = rs[((size_t)b * Hq + hq) * L + j];
  unsigned char* stage = smem + 32768;
  const int row = 32 * w + r32;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int d0 = 32 * dt + 8 * i4 + 4 * h;
      const bf16x4_t sv = *reinterpret_cast<const bf16x4_t*>(xs + roff + d0);
      const f32x4_t a = __builtin_convertvector(sv, f32x4_t);
      float4 g1 = make_float4(1.f, 1.f, 1.f, 1.f), g2 = g1;
      if (gs) g1 = *reinterpret_cast<const float4*>(gs + hq * 128 + d0);
      if (gr) g2 = *reinterpret_cast<const float4*>(gr + hq * 128 + d0);
      const f32x4_t val = {g1.x * a[0] * r_s + g2.x * acc[dt][4 * i4] * r_r, g1.y * a[1] * r_s + g2.y * acc[dt][4 * i4 + 1] * r_r,
                           g1.z * a[2] * r_s + g2.z * acc[dt][4 * i4 + 2] * r_r, g1.w * a[3] * r_s + g2.w * acc[dt][4 * i4 + 3] * r_r};
      const int c = 4 * dt + i4;
      *reinterpret_cast<bf16x4_t*>(stage + row * ROW_BYTES + ((c ^ swz(row)) << 4) + 8 * h) = __builtin_convertvector(val, bf16x4_t);
    }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = threadIdx.x + 256 * i;
    const int r = id >> 4, pch = id & 15;
    const int t = j0 + r - R;  // row of the chunk
    if (t >= 0) {
      const int c = pch ^ swz(r);
      *reinterpret_cast<uint4*>(o + ((size_t)(b * Tc + t) * Hq + hq) * 128 + c * 8) =
          *reinterpret_cast<const uint4*>(stage + r * ROW_BYTES + (pch << 4));
    }
  }
}

}  // namespace

void chunk_concat(const LayerDims& dmc, int dtype, int Tc, int R, int pos0, const void* q, const void* k, const void* v,
                  const void* k_ring, const void* v_ring, void* qc, void* kc, void* vc, hipStream_t st) {
  const int esize = dtype == 0 ? 4 : 2;
  const int row_vecs = dmc.D * esize / 16;
  const long long total = (long long)dmc.B * (R + Tc) * (dmc.Hkv + (q ? dmc.Hq : 0)) * row_vecs;
  const int blocks = (int)((total + 255) / 256 < 16384 ? (total + 255) / 256 : 16384);
  ProfScope ps("chunk_concat_kernel", st);
  chunk_concat_kernel<<<blocks, 256, 0, st>>>((const uint4*)q, (const uint4*)k, (const uint4*)v, (const uint4*)k_ring,
                                              (const uint4*)v_ring, (uint4*)qc, (uint4*)kc, (uint4*)vc, dmc.B, Tc, R,
                                              dmc.Hq, dmc.Hkv, dmc.W, pos0, row_vecs);
}

void chunk_copy_out(const LayerDims& dmc, int dtype, int Tc, int R, const void* oc, void* o, hipStream_t st) {
  const int esize = dtype == 0 ? 4 : 2;
  const long long rv = (long long)dmc.Hq * dmc.D * esize / 16;
  const long long total = (long long)dmc.B * Tc * rv;
  const int blocks = (int)((total + 255) / 256 < 16384 ? (total + 255) / 256 : 16384);
  ProfScope ps("chunk_copy_out_kernel", st);
  chunk_copy_out_kernel<<<blocks, 256, 0, st>>>((const uint4*)oc, (uint4*)o, dmc.B, Tc, R, rv);
}

void chunk_fixup(const LayerDims& dmc, int dtype, int Tc, int R, int Ls, const void* qc, const SavedPtrs& sv,
                 const float* state, const float* gs, const float* gr, void* o, hipStream_t st) {
  ProfScope ps("chunk_fixup_kernel", st);
  if (dtype == 1 && dmc.D == 128 && dmc.Dv == 128 && dmc.T % 128 == 0 && Ls == dmc.T && !sv.f32) {
    const dim3 tiles(dmc.T / 128 - R / 128, dmc.Hq, dmc.B);
#define RATTN_FIXUP_MFMA(FM_)                                                                                          \
  chunk_fixup_mfma_kernel<FM_><<<tiles, 256, 0, st>>>((const uint16_t*)qc, (const uint16_t*)sv.xs, (const uint16_t*)sv.xr, \
                                                      sv.rs, state, gs, gr, (uint16_t*)o, Tc, R, dmc.Hq, dmc.Hkv, dmc.eps)
    switch (feature_map_variant(dmc)) {
      case FM_RELU: RATTN_FIXUP_MFMA(FM_RELU); break;
      case FM_IDENTITY: RATTN_FIXUP_MFMA(FM_IDENTITY); break;
      default: RATTN_FIXUP_MFMA(FM_SOFTMAX); break;
    }
#undef RATTN_FIXUP_MFMA
    return;
  }
  const dim3 grid((Tc + 63) / 64, dmc.Hq, dmc.B);
  const size_t lds = (size_t)dmc.D * dmc.D * sizeof(float);
#define RATTN_FIXUP(IO, ST, DD)                                                                                      \
  chunk_fixup_kernel<IO, ST, DD><<<grid, 256, lds, st>>>((const IO*)qc, (const ST*)sv.xs, (const ST*)sv.xr, sv.rs, state, \
                                                         gs, gr, (IO*)o, Tc, R, Ls, dmc.Hq, dmc.Hkv, dmc.eps, dmc.phi)
  if (dtype == 0) {
    if (dmc.D == 64) RATTN_FIXUP(float, float, 64); else RATTN_FIXUP(float, float, 128);
  } else if (sv.f32) {
    if (dmc.D == 64) RATTN_FIXUP(bf16_t, float, 64); else RATTN_FIXUP(bf16_t, float, 128);
  } else {
    if (dmc.D == 64) RATTN_FIXUP(bf16_t, bf16_t, 64); else RATTN_FIXUP(bf16_t, bf16_t, 128);
  }
#undef RATTN_FIXUP
}

}  // namespace rattn
