// Device helpers for the gfx950 attention kernels: MFMA operand types, the swizzled LDS tile
// layout, and the two ways a 32x16 operand fragment is fetched from it.
//
// v_mfma_f32_32x32x16_bf16 register layout (lane l, g = l/32, n = l%32):
//   A (M x 16): row m = n,  k = 8g + j   (j = 0..7, one bf16x8 per lane)
//   B (16 x N): col n,      k = 8g + j
//   C (M x N):  col n,      row m = 8*(r/4) + 4g + r%4   (r = 0..15)
// A C-layout result can therefore be fed back as a B operand whose contraction index is the
// C row index, provided the other operand enumerates that index in the same order: for the
// 16-wide step t the lane group g holds C rows {16t + 4g + 0..3, 16t + 8 + 4g + 0..3}.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace peagle {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define PEAGLE_LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// LDS tile of `rows` x D bf16, row stride 2*D bytes.  The 16-byte chunk index of a row is
// XORed with a 3-bit function of the row so that (a) 8 consecutive rows read at the same
// logical chunk (ds_read_b128, lane <-> row) and (b) 4 consecutive rows read as 32-byte
// pairs (ds_read_b64_tr_b16) both spread over all banks.
__device__ __forceinline__ int swz3(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }

template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (2 * D) + ((chunk ^ swz3(row)) << 4);
}

// Natural fragment: lane <-> tile row (row0 + l%32), 8 consecutive elements along D starting
// at 16*step + 8g.  Serves as the A or B operand when the contraction runs over D.
template <int D>
__device__ __forceinline__ bf16x8 frag_nat(const char* tile, int row, int step, int g) {
  return *reinterpret_cast<const bf16x8*>(tile + tile_off<D>(row, 2 * step + g));
}

// Transposed fragment (ds_read_b64_tr_b16): lane <-> column (d0 + l%32) of the tile, the 8
// values run over tile rows {r0 + 4g + 0..3, r0 + 8 + 4g + 0..3}, r0 a multiple of 16.
// Within each group of 16 lanes the instruction returns to lane i element (i%4) of the 8-byte
// row segments addressed by lanes 4j + i/4 (j = 0..3): lane i supplies the address of row
// (i/4), column segment 4*(i%4) of its group's 16 columns.
struct TrLane {
  int row_in8;   // 4g + (l%16)/4 : row offset inside the 8-row half step
  int col;       // 16*((l/16)%2) + 4*(l%4) : first column (relative to d0) of the 8-byte segment
};
__device__ __forceinline__ TrLane tr_lane(int lane) {
  TrLane t;
  t.row_in8 = 4 * (lane >> 5) + ((lane & 15) >> 2);
  t.col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  return t;
}
template <int D>
__device__ __forceinline__ bf16x8 frag_tr(const char* tile, int r0, int d0, TrLane tl) {
  const int c = d0 + tl.col;  // element column
  const int row_a = r0 + tl.row_in8;
  const int row_b = row_a + 8;
  const int sw = swz3(row_a);  // same for row_b (differs by 8)
  const int off_in_row = (((c >> 3) ^ sw) << 4) + ((c & 7) << 1);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PEAGLE_LDS_PTR(s16x4, tile + row_a * (2 * D) + off_in_row));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PEAGLE_LDS_PTR(s16x4, tile + row_b * (2 * D) + off_in_row));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 p;
  p[0] = (__bf16)a;
  p[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, p);
}

// 8 consecutive C registers (one 16-wide contraction step) -> bf16x8 B operand.
__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int t) {
  u32x4 u;
  u[0] = pack_bf16(x[8 * t + 0], x[8 * t + 1]);
  u[1] = pack_bf16(x[8 * t + 2], x[8 * t + 3]);
  u[2] = pack_bf16(x[8 * t + 4], x[8 * t + 5]);
  u[3] = pack_bf16(x[8 * t + 6], x[8 * t + 7]);
  return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Value held by the lane 32 positions away (the other half of the same MFMA column).
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

}  // namespace peagle
