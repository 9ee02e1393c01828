// Chunk states of the linear branch for the MFMA paths (Eq. 2): chunk-local outer-product sums on the
// matrix cores, then an element-wise scan over chunks in fp32, stored as bf16 MFMA operands.
// States are kept transposed, [value feature d][phi feature f], because that is the row-major operand
// the consumers need.
#include "common.hpp"
#include "kernels.hpp"
#include "mfma.hpp"
#include <limits.h>

namespace rattn {

namespace {

struct ChunkArgs {
  const uint16_t* a;   // rows that go through phi  (k, or q for the reverse states)
  const uint16_t* b;   // rows multiplied in        (v, or dx_r)
  float* U;            // [B,Hkv,nchunks,128,128] fp32, U^T = B^T phi(A)
  // rows per sequence of a and of b as laid out in memory; rows >= Tfull_a / Tfull_b come from the 128-row tail
  // buffers instead (ragged lengths, see split_rows; INT_MAX and null when the tensor holds every row itself)
  const uint16_t *a_tail, *b_tail;
  int Ta, Tb, Tfull_a, Tfull_b;
  int H, GA;           // heads in a/b, heads summed per kv head
  int tok_off;         // token index = t' + tok_off
  int skip_m, skip_head, skip_per;  // skip_m > 1: product c leads from state i = (c - skip_head) / skip_per to i + 1 and is
                                    // left out when that state is a stored one ((i + 1) % skip_m == 0) or c < skip_head
  int first_lo, first_n, rest_lo, ckeys, tok_end;  // chunk 0 = [first_lo, +first_n); chunk c > 0 = ckeys tokens from
                                                   // rest_lo + ckeys (c-1); every chunk is clipped at tok_end
};

// grid (nchunks, Hkv, B), 256 threads.  Wave w owns rows d in [32w, 32w+32) of U^T.
template <int FM>
__global__ __launch_bounds__(256, 2) void rla_chunk_kernel(ChunkArgs p) {
  __shared__ __align__(16) unsigned char smem[65536];
  unsigned char* At = smem;
  unsigned char* Bt = smem + 32768;
  const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, nchunks = gridDim.x, Hkv = gridDim.y;
  if (p.skip_m > 1 && (c < p.skip_head || ((c - p.skip_head) / p.skip_per + 1) % p.skip_m == 0)) return;  // block-uniform
  const int lane = lane_id(), w = wave_id();
  const int r32 = lane & 31, h = lane >> 5;
  const int lo = c == 0 ? p.first_lo : p.rest_lo + p.ckeys * (c - 1);
  const int ntok = min(c == 0 ? p.first_n : p.ckeys, p.tok_end - lo);  // 64 or 128
  const size_t rstride = (size_t)p.H * 128;
  f32x16_t acc[4] = {{0}, {0}, {0}, {0}};
  for (int ga = 0; ga < p.GA; ++ga) {
    const int row = lo + p.tok_off, hd = g * p.GA + ga;   // chunks start at multiples of 64 rows
    if (ga > 0) __syncthreads();
    tile_load_async<4>(split_rows(p.a, p.a_tail, b, row, p.Ta, p.Tfull_a, p.H, hd), rstride, At, w * 4, lane);
    tile_load_async<4>(split_rows(p.b, p.b_tail, b, row, p.Tb, p.Tfull_b, p.H, hd), rstride, Bt, w * 4, lane);
    if (ntok == 128) {
      // rows 64..127 have their own source (they may be the ragged tail); the loader adds 64 row strides for these
      // blocks, so the base is given 64 rows back (never dereferenced there)
      const size_t back = (size_t)64 * rstride;
      tile_load_async<4>(split_rows(p.a, p.a_tail, b, row + 64, p.Ta, p.Tfull_a, p.H, hd) - back, rstride, At, 16 + w * 4, lane);
      tile_load_async<4>(split_rows(p.b, p.b_tail, b, row + 64, p.Tb, p.Tfull_b, p.H, hd) - back, rstride, Bt, 16 + w * 4, lane);
    }
    wait_vmem();
    __syncthreads();
    phi_tile_inplace<FM>(At, ntok);
    __syncthreads();
    // rolled on purpose: fully unrolled, the operand reads of all sub-blocks are hoisted and the kernel needs twice
    // the registers, which halves the work-groups per CU of a kernel that lives on memory-level parallelism
#pragma unroll 1
    for (int ks = 0; ks < ntok / 16; ++ks) {
      const int k0 = 16 * ks + 8 * h;
      const bf16x8_t aop = lds_tr_pair(Bt, k0, k0 + 4, 32 * w, lane);
#pragma unroll
      for (int ft = 0; ft < 4; ++ft) acc[ft] = mfma32(aop, lds_tr_pair(At, k0, k0 + 4, 32 * ft, lane), acc[ft]);
    }
  }
  float* out = p.U + ((size_t)(b * Hkv + g) * nchunks + c) * 16384;
#pragma unroll
  for (int ft = 0; ft < 4; ++ft)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int d = 32 * w + 8 * (i >> 2) + 4 * h + (i & 3);
      out[(size_t)d * 128 + 32 * ft + r32] = acc[ft][i];
    }
}

// Exclusive scan over chunks, every state element independently, fp32 accumulation, bf16 output.  A state spans
// PER chunk products (1, or 2 when the products cover 64 keys each).
//   forward: state[0] = sum of the `head` products in front of it; state[i+1] = state[i] + the next `per` products
//   reverse: state[n-1] = 0; state[i] = state[i+1] + products per*i .. per*i + per - 1 (those that exist)
// grid (16, Hkv, B), 256 threads, 4 elements per thread.
// init (forward only, may be NULL): a state that precedes chunk 0, fp32 [B,Hkv,f,d] (not transposed).
// Forward scan with m > 1: `subset` (may be NULL) also receives states 0, m, 2m, ... ([B,Hkv,ceil(nst/m),128,128]);
// `restart` (may be NULL) holds such a subset, and the running sum is replaced by the stored state at every multiple
// of m (the products that lead to a stored state are then never used and need not exist).
template <bool REV, int PER>
__global__ __launch_bounds__(256) void rla_scan_kernel(const float* __restrict__ U, uint16_t* __restrict__ states,
                                                       int nchunks, int nst, int head,
                                                       const float* __restrict__ init, uint16_t* __restrict__ subset,
                                                       const uint16_t* __restrict__ restart, int m) {
  const int g = blockIdx.y, b = blockIdx.z, Hkv = gridDim.y;
  const int e4 = (blockIdx.x * 256 + threadIdx.x) * 4;
  const float* Ub = U + (size_t)(b * Hkv + g) * nchunks * 16384 + e4;
  uint16_t* Sb = states + (size_t)(b * Hkv + g) * nst * 16384 + e4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (!REV && init) {  // element (d, f .. f+3) of the transposed state = init[f .. f+3][d]
    const float* ib = init + (size_t)(b * Hkv + g) * 16384 + (e4 >> 7);
    const int f = e4 & 127;
    acc = make_float4(ib[(size_t)f * 128], ib[(size_t)(f + 1) * 128], ib[(size_t)(f + 2) * 128], ib[(size_t)(f + 3) * 128]);
  }
  const int nsub = (!REV && m > 1) ? (nst + m - 1) / m : 0;
  const size_t sub0 = (size_t)(b * Hkv + g) * nsub * 16384 + e4;
  auto put = [&](int i) {
    if (!REV && restart && i % m == 0) {  // continue from the state the forward pass stored
      const bf16x4_t s = *reinterpret_cast<const bf16x4_t*>(restart + sub0 + (size_t)(i / m) * 16384);
      acc = make_float4((float)s[0], (float)s[1], (float)s[2], (float)s[3]);
    }
    f32x4_t f = {acc.x, acc.y, acc.z, acc.w};
    const bf16x4_t o = __builtin_convertvector(f, bf16x4_t);
    *reinterpret_cast<bf16x4_t*>(Sb + (size_t)i * 16384) = o;
    if (!REV && subset && i % m == 0) *reinterpret_cast<bf16x4_t*>(subset + sub0 + (size_t)(i / m) * 16384) = o;
  };
  auto ld = [&](int c) {  // product c, or zero when it does not exist
    return (c >= 0 && c < nchunks) ? *reinterpret_cast<const float4*>(Ub + (size_t)c * 16384) : make_float4(0.f, 0.f, 0.f, 0.f);
  };
  auto add = [&](const float4& u) { acc.x += u.x; acc.y += u.y; acc.z += u.z; acc.w += u.w; };
  // States are walked in groups of GRP: the group's products are all requested before the first is added, so the
  // loads of a group are in flight together (the additions keep their fixed order).
  constexpr int GRP = 4;
  if (!REV) {
    if (!restart)
      for (int c = 0; c < head; ++c) add(ld(c));
    // state i is stored, then products head + PER*i .. + PER - 1 are added to reach state i + 1
    for (int i0 = 0; i0 < nst; i0 += GRP) {
      float4 u[GRP][PER];
#pragma unroll
      for (int j = 0; j < GRP; ++j)
#pragma unroll
        for (int r = 0; r < PER; ++r) u[j][r] = (i0 + j + 1 < nst && !(restart && (i0 + j + 1) % m == 0)) ? ld(head + PER * (i0 + j) + r) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int j = 0; j < GRP; ++j) {
        if (i0 + j < nst) put(i0 + j);
#pragma unroll
        for (int r = 0; r < PER; ++r) add(u[j][r]);
      }
    }
  } else {
    // state nst-1 = 0; state i = state i+1 + products PER*i .. PER*i + PER - 1 (descending order of addition)
    for (int i0 = nst - 1; i0 >= 0; i0 -= GRP) {
      float4 u[GRP][PER];
#pragma unroll
      for (int j = 0; j < GRP; ++j)
#pragma unroll
        for (int r = 0; r < PER; ++r) u[j][r] = (i0 - j > 0) ? ld(PER * (i0 - j - 1) + r) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int j = 0; j < GRP; ++j) {
        if (i0 - j >= 0) put(i0 - j);
#pragma unroll
        for (int r = PER - 1; r >= 0; --r) add(u[j][r]);
      }
    }
  }
}

void launch_chunk_kernel(int fm, dim3 grid, const ChunkArgs& p, hipStream_t st) {
  switch (fm) {
    case FM_RELU: rla_chunk_kernel<FM_RELU><<<grid, 256, 0, st>>>(p); break;
    case FM_IDENTITY: rla_chunk_kernel<FM_IDENTITY><<<grid, 256, 0, st>>>(p); break;
    case FM_SOFTMAX64: rla_chunk_kernel<FM_SOFTMAX64><<<grid, 256, 0, st>>>(p); break;
    default: rla_chunk_kernel<FM_SOFTMAX><<<grid, 256, 0, st>>>(p); break;
  }
}

}  // namespace

void rla_forward_states(const LayerDims& dm, const FastFwdPlan& pl, const void* k, const void* v, float* U,
                        void* states, hipStream_t st, const float* state0, const RaggedTails* tails, void* subset_out,
                        const void* restart, int m) {
  if (pl.nstf <= 0) return;
  if (m < 2) { m = 1; subset_out = nullptr; restart = nullptr; }
  const int head = pl.base > 0 ? 1 : 0;  // products in front of state 0: the 64 keys before it when it sits at key 64
  if (pl.nchunks > 0) {
    ChunkArgs p;
    p.a = (const uint16_t*)k; p.b = (const uint16_t*)v; p.U = U;
    p.a_tail = tails ? (const uint16_t*)tails->k : nullptr; p.b_tail = tails ? (const uint16_t*)tails->v : nullptr;
    p.Ta = p.Tb = tails ? tails->Tc : dm.T;
    p.Tfull_a = p.Tfull_b = tails ? tails->Tc / 128 * 128 : INT_MAX;
    p.H = dm.Hkv; p.GA = 1; p.tok_off = 0;
    p.ckeys = pl.ckeys;
    p.first_lo = 0; p.first_n = head ? 64 : pl.ckeys; p.rest_lo = p.first_n; p.tok_end = 1 << 30;
    p.skip_m = restart ? m : 0; p.skip_head = head; p.skip_per = 128 / pl.ckeys;
    ProfScope ps("rla_chunk_kernel", st);
    launch_chunk_kernel(feature_map_variant(dm), dim3(pl.nchunks, dm.Hkv, dm.B), p, st);
  }
  ProfScope ps("rla_scan_kernel", st);
  const dim3 sgrid(16, dm.Hkv, dm.B);
  if (pl.ckeys == 64)
    rla_scan_kernel<false, 2><<<sgrid, 256, 0, st>>>(U, (uint16_t*)states, pl.nchunks, pl.nstf, head, state0,
                                                     (uint16_t*)subset_out, (const uint16_t*)restart, m);
  else
    rla_scan_kernel<false, 1><<<sgrid, 256, 0, st>>>(U, (uint16_t*)states, pl.nchunks, pl.nstf, head, state0,
                                                     (uint16_t*)subset_out, (const uint16_t*)restart, m);
}

void rla_reverse_states(const LayerDims& dm, const FastBwdPlan& pl, const void* q, const void* dxr, float* U,
                        void* rstates, hipStream_t st, const RaggedTails* tails) {
  if (pl.nk <= 0) return;
  const int W = pl.fwd.W, Tp = dm.T - W, ck = pl.fwd.ckeys;
  if (pl.nrchunks > 0) {
    ChunkArgs p;
    p.a = (const uint16_t*)q; p.b = (const uint16_t*)dxr; p.U = U;
    p.a_tail = tails ? (const uint16_t*)tails->q : nullptr; p.b_tail = nullptr;   // dx_r is a workspace tensor
    p.Ta = tails ? tails->Tc : dm.T; p.Tb = dm.T;
    p.Tfull_a = tails ? tails->Tc / 128 * 128 : INT_MAX; p.Tfull_b = INT_MAX;
    p.H = dm.Hq; p.GA = dm.G; p.tok_off = W;
    p.ckeys = ck;
    p.first_lo = 128; p.first_n = ck; p.rest_lo = 128 + ck; p.tok_end = Tp;
    p.skip_m = 0; p.skip_head = 0; p.skip_per = 1;
    ProfScope ps("rla_chunk_kernel(rev)", st);
    launch_chunk_kernel(feature_map_variant(dm), dim3(pl.nrchunks, dm.Hkv, dm.B), p, st);
  }
  ProfScope ps("rla_scan_kernel(rev)", st);
  const dim3 sgrid(16, dm.Hkv, dm.B);
  if (ck == 64) rla_scan_kernel<true, 2><<<sgrid, 256, 0, st>>>(U, (uint16_t*)rstates, pl.nrchunks, pl.nk, 0, nullptr, nullptr, nullptr, 1);
  else rla_scan_kernel<true, 1><<<sgrid, 256, 0, st>>>(U, (uint16_t*)rstates, pl.nrchunks, pl.nk, 0, nullptr, nullptr, nullptr, 1);
}

}  // namespace rattn
