// Building blocks for the bf16 MFMA kernels on gfx950 (CDNA4): vector types, the
// v_mfma_f32_32x32x16_bf16 wrapper with its register layouts, and the LDS tile layout.
//
// v_mfma_f32_32x32x16_bf16 computes C[32x32] += A[32x16] B[16x32] per wavefront.  With
// lane l, r = l % 32, h = l / 32:
//   A operand (8 bf16): A[r][8h .. 8h+7]         B operand (8 bf16): B[8h .. 8h+7][r]
//   C/D (16 fp32):      C[(i/4)*8 + 4h + i%4][r] for i = 0..15
// Because the contraction index only has to match between A and B, a C tile can be fed
// back as the B operand of the next product without any data movement: the 8 values
// C[.][r] with i in [8u, 8u+8) become B[8h+e][r], provided the A operand of that product is
// gathered with the same row order, rows (e/4)*8 + 4h + e%4 of the 16-row block u.
//
// LDS tiles hold rows of 128 bf16 (256 B, sixteen 16-byte chunks) without padding; chunk c
// of row r is stored at chunk position c ^ swz(r).  With swz(r) = ((r&3)<<2) | ((r>>2)&3)
// both access patterns used here are bank-conflict free: ds_read_b128 of one chunk column
// from 16 consecutive rows, and ds_read_b64_tr_b16 of 4 rows x 64 B.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dfa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define DFA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// byte offset of 16-byte chunk c of row r inside a 256-B-per-row tile
__device__ __forceinline__ int tile_off(int r, int c) { return r * 256 + ((c ^ swz(r)) << 4); }

__device__ __forceinline__ bf16x8 lds_read_b128(const char* base, int off) {
  return *reinterpret_cast<const bf16x8*>(base + off);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane j supplies
// the address of 4 consecutive bf16; lane i receives, for t = 0..3, element (i % 4) of the
// 4 that lane (4t + i/4) of its group addressed.
__device__ __forceinline__ bf16x4 lds_read_tr(const char* base, int off) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (DFA_LDS s16x4*)(base + off));
  return __builtin_bit_cast(bf16x4, v);
}

// 8 values for the A operand of a product whose contraction runs over tile ROWS (the tile is
// stored row-major, so this is a transposed gather): rows row0 + (e/4)*8 + 4h + e%4, column
// col0 + (lane % 32).  row0 must be a multiple of 16, col0 a multiple of 32.
__device__ __forceinline__ bf16x8 lds_gather_rows(const char* base, int row0, int col0, int lane) {
  const int g = lane >> 4, j = lane & 15;
  const int row = row0 + 4 * (g >> 1) + (j >> 2);
  const int c = (col0 >> 3) + 2 * (g & 1) + ((j & 3) >> 1);
  const int sub = (j & 1) << 3;
  const bf16x4 lo = lds_read_tr(base, tile_off(row, c) + sub);
  const bf16x4 hi = lds_read_tr(base, tile_off(row + 8, c) + sub);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = static_cast<__bf16>(v[first + e]);
  return r;
}

}  // namespace dfa
