// gfx950 matrix-core and LDS helpers shared by the MFMA kernels.
//
// v_mfma_f32_32x32x16_bf16 operand layout (wave of 64 lanes, lane = 32*h + r):
//   A (32 x 16): lane holds row r, contraction slots 8h..8h+7 (8 bf16 in 4 VGPRs)
//   B (16 x 32): lane holds column r, contraction slots 8h..8h+7
//   C (32 x 32): lane holds column r; register i (0..15) is row 8*(i/4) + 4h + i%4
// ds_read_b64_tr_b16 (16-lane groups): if source lane 4j+c of a group points at M[k0+j][n0+4c..+3],
//   lane i of the group receives M[k0+0..3][n0+i]: a 4(k) x 16(n) block of a row-major matrix is
//   delivered k-contiguous per lane, which is what an MFMA operand wants when memory is n-contiguous.
// Tiles in LDS are rows of 128 bf16 (256 bytes = 16 chunks of 16 bytes); the chunk index is XOR-swizzled
// with swz(row) = ((row & 3) << 2) | ((row >> 2) & 3) so that both access patterns are bank-conflict free
// without padding:
//   row reads (ds_read_b128, 16 lanes on 16 consecutive rows, same logical chunk): swz takes 16 values
//   tr reads  (ds_read_b64_tr_b16, 4 consecutive rows x 64 bytes per half-wave): the upper two bits of
//             swz differ between the 4 rows, so the four 64-byte pieces land in different bank groups
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rattn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

#define RATTN_LDS(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int ROW_BYTES = 256;  // 128 bf16

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ f32x16_t mfma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// wait until every outstanding vector-memory operation of this wave (incl. direct-to-LDS loads) is done
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// 16 bytes per lane from global memory straight into LDS at lds_addr + 16*lane (lds_addr wave-uniform).
// Issued through inline assembly on purpose: the compiler then does not put its own conservative
// vmcnt waits in front of later LDS reads, so a tile prefetch really overlaps the math on the current
// tile; completion is awaited explicitly with wait_vmem() before the barrier that publishes the tile.
__device__ __forceinline__ void dma16(const void* g, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory", "m0");
}

// Asynchronously copy `NBLK` blocks of 4 rows x 256 bytes from global memory into an LDS tile, direct to
// LDS (no VGPR staging).  Block index blk0 + i, lane l lands at tile + blk*1024 + l*16, i.e. row
// 4*blk + l/16, physical chunk l%16; it fetches the logical chunk that the swizzle maps there.
template <int NBLK>
__device__ __forceinline__ void tile_load_async(const uint16_t* gbase, size_t row_stride, unsigned char* tile,
                                                int blk0, int lane) {
#pragma unroll
  for (int i = 0; i < NBLK; ++i) {
    const int blk = blk0 + i;
    const int r = blk * 4 + (lane >> 4);
    const int p = lane & 15;
    const int c = p ^ swz(r);
    const uint16_t* g = gbase + (size_t)r * row_stride + c * 8;
    dma16(g, (unsigned)(size_t)RATTN_LDS(tile + blk * 1024));
  }
}

// The same load with a wave-uniform base in scalar registers and a 32-bit per-lane byte offset: no per-lane 64-bit
// address arithmetic per load.
__device__ __forceinline__ void dma16s(const void* sbase, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory", "m0");
}
// Per-lane byte offsets of tile_load_async's access pattern inside a 4-row block, one per value of (block & 3)
// (the swizzle of row 4*blk + lane/16 depends on the block only through blk & 3); computed once per kernel.
struct DmaLane { unsigned off[4]; };
__device__ __forceinline__ DmaLane make_dma_lane(int lane, size_t row_stride_elems) {
  DmaLane d;
  const int l4 = lane >> 4, p = lane & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) d.off[i] = (unsigned)(l4 * row_stride_elems * 2) + (unsigned)((p ^ ((l4 << 2) | i)) << 4);
  return d;
}
// tile_load_async for NBLK consecutive blocks starting at blk0 (a multiple of 4, wave-uniform), NBLK <= 4... 8
template <int NBLK>
__device__ __forceinline__ void tile_load_async_s(const uint16_t* gbase, size_t row_stride, unsigned char* tile, int blk0,
                                                  const DmaLane& dl) {
#pragma unroll
  for (int i = 0; i < NBLK; ++i) {
    const int blk = blk0 + i;
    dma16s(gbase + (size_t)blk * 4 * row_stride, dl.off[i & 3], (unsigned)(size_t)RATTN_LDS(tile + blk * 1024));
  }
}

// operand whose rows are tile rows: 8 consecutive elements at logical chunk c of row r
__device__ __forceinline__ bf16x8_t lds_row_chunk(const unsigned char* tile, int r, int c) {
  return *reinterpret_cast<const bf16x8_t*>(tile + r * ROW_BYTES + ((c ^ swz(r)) << 4));
}

// operand whose rows are tile COLUMNS.  Lane (r = lane%32, h = lane/32) receives
// tile[ka + 0..3][col0 + r] and tile[kb + 0..3][col0 + r]  (ka, kb multiples of 4, per-lane values allowed
// as long as they are equal within each 16-lane group), col0 a multiple of 32.
__device__ __forceinline__ bf16x8_t lds_tr_pair(const unsigned char* tile, int ka, int kb, int col0, int lane) {
  const int i = lane & 15, gi = lane >> 4;
  const int j = i >> 2;
  const int c = (col0 >> 3) + 2 * (gi & 1) + ((i & 3) >> 1);
  const int boff = (i & 1) << 3;
  const int ra = ka + j, rb = kb + j;
  const unsigned char* pa = tile + ra * ROW_BYTES + ((c ^ swz(ra)) << 4) + boff;
  const unsigned char* pb = tile + rb * ROW_BYTES + ((c ^ swz(rb)) << 4) + boff;
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(pa));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(pb));
  union { struct { s16x4_t lo, hi; } s; bf16x8_t v; } u;
  u.s.lo = lo; u.s.hi = hi;
  return u.v;
}

// Per-lane LDS byte offsets, computed once per kernel so that the hot loops issue ds_read with a
// register offset plus an immediate (the XOR swizzle is not affine, the compiler cannot fold it).
struct LaneOff {
  int row[8];     // row read: logical chunk 2*c2 + h of row (lane % 32)
  int trp[4][2];  // transposed read, contraction slots in accumulator order: rows 4h + 8*ab + (0..3), columns 32*ct + lane%32
};
struct LaneOffN {
  int trn[4][2];  // transposed read, natural contraction order: rows 8h + 4*ab + (0..3), columns 32*ct + lane%32
};
__device__ __forceinline__ int tr_lane_off(int rl, int ct, int lane) {
  const int i = lane & 15, gi = lane >> 4;
  const int r = rl + (i >> 2);
  const int c = 4 * ct + 2 * (gi & 1) + ((i & 3) >> 1);
  return r * ROW_BYTES + ((c ^ swz(r)) << 4) + ((i & 1) << 3);
}
__device__ __forceinline__ LaneOff make_lane_off(int lane) {
  LaneOff lo;
  const int r32 = lane & 31, h = lane >> 5;
#pragma unroll
  for (int c2 = 0; c2 < 8; ++c2) lo.row[c2] = r32 * ROW_BYTES + (((2 * c2 + h) ^ swz(r32)) << 4);
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int ab = 0; ab < 2; ++ab) lo.trp[ct][ab] = tr_lane_off(4 * h + 8 * ab, ct, lane);
  return lo;
}
__device__ __forceinline__ LaneOffN make_lane_off_n(int lane) {
  LaneOffN lo;
  const int h = lane >> 5;
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int ab = 0; ab < 2; ++ab) lo.trn[ct][ab] = tr_lane_off(8 * h + 4 * ab, ct, lane);
  return lo;
}
// A/B operand = rows R0 + lane%32 of the tile (R0 % 16 == 0), elements 16*c2 + 8h .. +7
__device__ __forceinline__ bf16x8_t lds_row(const unsigned char* tile, const LaneOff& lo, int R0, int c2) {
  return *reinterpret_cast<const bf16x8_t*>(tile + lo.row[c2] + R0 * ROW_BYTES);
}
__device__ __forceinline__ bf16x8_t lds_tr2(const unsigned char* pa, const unsigned char* pb) {
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(pa));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(pb));
  union { struct { s16x4_t lo, hi; } s; bf16x8_t v; } u;
  u.s.lo = lo; u.s.hi = hi;
  return u.v;
}
// operand = columns 32*ct + lane%32 of the tile; slot e of half h is tile row K0 + 8(e/4) + 4h + e%4
// (the order in which a 32x32 accumulator holds its rows), K0 % 16 == 0
__device__ __forceinline__ bf16x8_t lds_trp(const unsigned char* tile, const LaneOff& lo, int K0, int ct) {
  return lds_tr2(tile + lo.trp[ct][0] + K0 * ROW_BYTES, tile + lo.trp[ct][1] + K0 * ROW_BYTES);
}
// same with natural order: slot e of half h is tile row K0 + 8h + e, K0 % 16 == 0
__device__ __forceinline__ bf16x8_t lds_trn(const unsigned char* tile, const LaneOffN& lo, int K0, int ct) {
  return lds_tr2(tile + lo.trn[ct][0] + K0 * ROW_BYTES, tile + lo.trn[ct][1] + K0 * ROW_BYTES);
}

__device__ __forceinline__ bf16x8_t pack_bf16x8(const float* x) {
  f32x8_t v = {x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7]};
  return __builtin_convertvector(v, bf16x8_t);
}

__device__ __forceinline__ void unpack_bf16x8(bf16x8_t v, float* x) {
  f32x8_t f = __builtin_convertvector(v, f32x8_t);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = f[i];
}

// combine a value with the one held by lane ^ 32 (v_permlane32_swap: one VALU op, no LDS traffic)
__device__ __forceinline__ float half_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// 2^x on the transcendental unit (v_exp_f32): 2^-inf = 0, no denormal fix-up code
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Ragged sequence lengths.  The kernels work on whole 128-row tiles of a padded length; a caller tensor [B, Tc, H, 128]
// whose length Tc is not a whole number of tiles is read (or written) in two parts: rows below Tfull = 128 * (Tc / 128)
// in place, the last, partial tile through a zero-padded 128-row copy [B, 128, H, 128] in the workspace.  A tile or
// half tile never straddles Tfull.  Without a ragged tail, Tfull is INT_MAX and the tail pointer is never used.
template <typename P>
__device__ __forceinline__ P* split_rows(P* main, P* tail, int b, int row, int Tc, int Tfull, int H, int h) {
  return row < Tfull ? main + ((size_t)(b * (size_t)Tc + row) * H + h) * 128
                     : tail + ((size_t)(b * (size_t)128 + (row - Tfull)) * H + h) * 128;
}

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Feature map of the linear branch as a compile-time choice of the matrix-core kernels:
//   FM_SOFTMAX    softmax over the 128 features of a row (Sec. 3.1)
//   FM_RELU       max(x, 0) per feature, FM_IDENTITY  x itself (the ablation's maps, Sec. 4.5)
//   FM_SOFTMAX64  softmax over the FIRST 64 features; features 64..127 are padding (the caller's head size is 64 and
//                 rows arrive zero-padded to 128): their phi is 0, so they drop out of every product.  The other two
//                 maps need no such variant: they map a padding zero to zero by themselves.
enum { FM_SOFTMAX = 0, FM_RELU = 1, FM_IDENTITY = 2, FM_SOFTMAX64 = 3 };

// phi of a row whose two halves sit in lanes l and l^32 (64 values each: x[8c + e] = feature 16c + 8h + e);
// result packed as 8 MFMA operand registers in the same order.
template <int FM = FM_SOFTMAX>
__device__ __forceinline__ void phi_rows(float (&x)[64], bf16x8_t (&op)[8]) {
  if (FM == FM_RELU) {
#pragma unroll
    for (int i = 0; i < 64; ++i) x[i] = fmaxf(x[i], 0.f);
  } else if (FM == FM_SOFTMAX || FM == FM_SOFTMAX64) {
    constexpr int NV = FM == FM_SOFTMAX64 ? 32 : 64;  // this lane's valid features: c < 4 are features < 64
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
#pragma unroll
  for (int c = 0; c < 8; ++c) op[c] = pack_bf16x8(&x[8 * c]);
}

// phi applied in place to LDS tile rows, two threads per row: thread pair r works on row r of tile A
// (r < 64) or row r-64 of tile B (r >= 64); a null tile pointer skips that half.  Tiles A and B
// contiguous = one 128-row tile.  Call with all 256 threads; the caller synchronises before and after.
template <int FM = FM_SOFTMAX>
__device__ __forceinline__ void phi_tiles_inplace(unsigned char* tileA, unsigned char* tileB) {
  if (FM == FM_IDENTITY) return;
  const int r = threadIdx.x >> 1, half = threadIdx.x & 1;
  unsigned char* tile = r < 64 ? tileA : tileB;
  const int row = r & 63;
  // FM_SOFTMAX64: the thread with features 64..127 has nothing to do (padding zeros stay zeros)
  if (tile && !(FM == FM_SOFTMAX64 && half == 1)) {
    float x[64];
    unsigned char* rp = tile + row * ROW_BYTES;
    const int sw = swz(row);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      unpack_bf16x8(*reinterpret_cast<const bf16x8_t*>(rp + (((8 * half + j) ^ sw) << 4)), &x[8 * j]);
    if (FM == FM_RELU) {
#pragma unroll
      for (int i = 0; i < 64; ++i) x[i] = fmaxf(x[i], 0.f);
    } else {
      float m = x[0];
#pragma unroll
      for (int i = 1; i < 64; ++i) m = fmaxf(m, x[i]);
      if (FM == FM_SOFTMAX) m = fmaxf(m, __shfl_xor(m, 1, 64));
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 64; ++i) { x[i] = fast_exp2((x[i] - m) * LOG2E); s += x[i]; }
      if (FM == FM_SOFTMAX) s += __shfl_xor(s, 1, 64);
      const float inv = 1.f / s;
#pragma unroll
      for (int i = 0; i < 64; ++i) x[i] *= inv;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      *reinterpret_cast<bf16x8_t*>(rp + (((8 * half + j) ^ sw) << 4)) = pack_bf16x8(&x[8 * j]);
  }
}
// first `nrows` (64 or 128) rows of one contiguous tile
template <int FM = FM_SOFTMAX>
__device__ __forceinline__ void phi_tile_inplace(unsigned char* tile, int nrows) {
  phi_tiles_inplace<FM>(tile, nrows > 64 ? tile + 64 * ROW_BYTES : nullptr);
}

// Write a [128 rows x 128] bf16 tile held transposed in accumulators (lane = tile row 32w + lane%32,
// register (dt,i) = column 32dt + 8(i/4) + 4h + i%4) to global rows of stride `row_stride`, through
// LDS so that the global stores are 16 bytes per lane and row-contiguous.  All 256 threads call it;
// smem[0..32K) is used and is free again on return.
__device__ __forceinline__ void store_tile_transposed(unsigned char* smem, const float (&vals)[4][16], uint16_t* dst,
                                                      size_t row_stride, int w, int lane) {
  const int r32 = lane & 31, h = lane >> 5;
  const int row = 32 * w + r32;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      f32x4_t f = {vals[dt][4 * i4], vals[dt][4 * i4 + 1], vals[dt][4 * i4 + 2], vals[dt][4 * i4 + 3]};
      bf16x4_t pk = __builtin_convertvector(f, bf16x4_t);
      const int c = 4 * dt + i4;
      *reinterpret_cast<bf16x4_t*>(smem + row * ROW_BYTES + ((c ^ swz(row)) << 4) + 8 * h) = pk;
    }
  __syncthreads();
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = tid + 256 * i;
    const int r = id >> 4, p = id & 15;
    const int c = p ^ swz(r);
    const u32x4_t val = *reinterpret_cast<const u32x4_t*>(smem + r * ROW_BYTES + (p << 4));
    // written once, not read again by the kernel that writes it: keep it from displacing the shared K/V tiles in L2
    __builtin_nontemporal_store(val, reinterpret_cast<u32x4_t*>(dst + (size_t)r * row_stride + c * 8));
  }
  __syncthreads();
}

}  // namespace rattn
