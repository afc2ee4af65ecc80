// Pieces shared by the bf16 MFMA attention kernels (forward and training backward): how 32x32x16 operands are laid
// out in LDS tiles and fetched from them, and the two-lane / wave reductions those kernels use.
//
// Conventions (v_mfma_f32_32x32x16_bf16, wave64; lane = 32*hb + c):
//   * a lane owns accumulator column c; its 16 registers are rows 8*(r/4) + 4*hb + r%4 of the product;
//   * tiles whose rows feed the A operand row-wise are stored padded (row stride D + 8 elements) and MFMA row m is
//     made to carry tile row tile_row_of_mfma_row(m), so that accumulator register r of lane half hb belongs to tile
//     row 16*(r/8) + 8*hb + r%8: a lane's eight values per MFMA are then eight consecutive tile rows, which is the
//     order the second product consumes them in as its B operand;
//   * tiles that feed the A operand transposed (contraction over tile rows) stay row-major and unpadded; their
//     64-byte chunks are XOR-swizzled with the row so that the transposing loads and the staging stores spread over
//     all banks.
#pragma once
#include "ltea_common.h"

namespace ltea {

// Swap bits 2 and 3 of m.
__device__ __forceinline__ int tile_row_of_mfma_row(int m) { return (m & 0x13) | ((m & 0x08) >> 1) | ((m & 0x04) << 1); }

// Which 64-byte chunk of its row a tile row's chunk c is stored in (c ^ term).  Four consecutive rows must land in
// four different 64-byte bank groups: rows are 128 bytes (D = 64, two chunks, alternate every second row) or 256
// bytes (D = 128, four chunks, rotate every row).
template <int D> __device__ __forceinline__ int chunk_swizzle(int row) { return D == 64 ? ((row >> 1) & 1) : (row & 3); }

// A operand from a row-major tile read transposed: eight consecutive tile rows of one column per lane, as two
// transposing 64-bit LDS loads (rows +0..3, +4..7).  In each group of 16 lanes, lane j points at the four columns
// c0 + 4*(j%4).. of tile row r0 + j/4 and receives column c0 + j of the four rows r0 .. r0+3.
__device__ __forceinline__ bf16x8 load_transposed(const bf16_t* p, int row_stride) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * row_stride));
  s16x8 r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return __builtin_bit_cast(bf16x8, r);
}

// Both lane halves (l, l^32) receive max / sum of the pair.
__device__ __forceinline__ float pair_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ int wave_min_i(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { const int y = __shfl_xor(x, off, kWave); x = y < x ? y : x; }
  return x;
}
__device__ __forceinline__ int wave_max_i(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { const int y = __shfl_xor(x, off, kWave); x = y > x ? y : x; }
  return x;
}

}  // namespace ltea
