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
// with the row so that both access patterns are bank-conflict free without padding:
//   "row" swizzle  (operand rows read with ds_read_b128, 16 lanes on 16 consecutive rows): chunk ^ (row & 15)
//   "tr" swizzle   (operand read with ds_read_b64_tr_b16, 4 consecutive rows x 64 bytes): chunk ^ ((row & 3) << 2)
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

#define RATTN_LDS(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int ROW_BYTES = 256;  // 128 bf16

__device__ __forceinline__ f32x16_t mfma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// wait until every outstanding vector-memory operation of this wave (incl. direct-to-LDS loads) is done
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Asynchronously copy `NBLK` blocks of 4 rows x 256 bytes from global memory into an LDS tile, direct to
// LDS (no VGPR staging).  Block index blk0 + i, lane l lands at tile + blk*1024 + l*16, i.e. row
// 4*blk + l/16, physical chunk l%16; it fetches the logical chunk that the swizzle maps there.
template <bool TR_SWZ, int NBLK>
__device__ __forceinline__ void tile_load_async(const uint16_t* gbase, size_t row_stride, unsigned char* tile,
                                                int blk0, int lane) {
#pragma unroll
  for (int i = 0; i < NBLK; ++i) {
    const int blk = blk0 + i;
    const int r = blk * 4 + (lane >> 4);
    const int p = lane & 15;
    const int c = TR_SWZ ? (p ^ ((r & 3) << 2)) : (p ^ (r & 15));
    const uint16_t* g = gbase + (size_t)r * row_stride + c * 8;
    __builtin_amdgcn_global_load_lds(g, RATTN_LDS(tile + blk * 1024), 16, 0, 0);
  }
}

// operand whose rows are tile rows ("row" swizzle): 8 consecutive elements at logical chunk c of row r
__device__ __forceinline__ bf16x8_t lds_row_chunk(const unsigned char* tile, int r, int c) {
  return *reinterpret_cast<const bf16x8_t*>(tile + r * ROW_BYTES + ((c ^ (r & 15)) << 4));
}

// operand whose rows are tile COLUMNS ("tr" swizzle).  Lane (r = lane%32, h = lane/32) receives
// tile[ka + 0..3][col0 + r] and tile[kb + 0..3][col0 + r]  (ka, kb multiples of 4, per-lane values allowed
// as long as they are equal within each 16-lane group), col0 a multiple of 32.
__device__ __forceinline__ bf16x8_t lds_tr_pair(const unsigned char* tile, int ka, int kb, int col0, int lane) {
  const int i = lane & 15, gi = lane >> 4;
  const int j = i >> 2;
  const int c = (col0 >> 3) + 2 * (gi & 1) + ((i & 3) >> 1);
  const int boff = (i & 1) << 3;
  const int ra = ka + j, rb = kb + j;
  const unsigned char* pa = tile + ra * ROW_BYTES + ((c ^ ((ra & 3) << 2)) << 4) + boff;
  const unsigned char* pb = tile + rb * ROW_BYTES + ((c ^ ((rb & 3) << 2)) << 4) + boff;
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(pa));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(pb));
  union { struct { s16x4_t lo, hi; } s; bf16x8_t v; } u;
  u.s.lo = lo; u.s.hi = hi;
  return u.v;
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

// value of the same register in lane ^ 32
__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32, 64); }

}  // namespace rattn
