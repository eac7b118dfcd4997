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

// LDS tile of `rows` x D bf16, row stride 2*D bytes.  The LDS of gfx950 has 64 banks of 4 bytes
// (256 B per clock): a ds_read_b128 is conflict-free when 16 consecutive lanes cover sixteen
// distinct 16-byte slots modulo 256 B, a ds_read_b64_tr_b16 when its 4 rows x 64 B do.  The
// 16-byte chunk index of a row is therefore XORed with a function of the row (period 16 rows)
// chosen so that both hold for the two fragment reads below:
//   D = 64  (two rows per 256 B): k = (row/2)%8, swz = (k%2)*4 + k/2
//   D = 128 (one row per 256 B):  swz = (row%4)*4 + (row/4)%4
template <int D>
__device__ __forceinline__ int swz(int row) {
  if (D == 64) {
    const int k = (row >> 1) & 7;
    return ((k & 1) << 2) | (k >> 1);
  }
  return ((row & 3) << 2) | ((row >> 2) & 3);
}

template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (2 * D) + ((chunk ^ swz<D>(row)) << 4);
}

// Natural fragment: lane <-> tile row (row0 + l%32), 8 consecutive elements along D starting
// at 16*step + 8g.  Serves as the A or B operand when the contraction runs over D.
// NatOff holds the per-lane byte offsets of the D/16 steps for row l%32; rows 32 apart share
// the swizzle, so other 32-row blocks add a compile-time constant.
template <int D>
struct NatOff {
  int off[D / 16];
};
template <int D>
__device__ __forceinline__ NatOff<D> nat_offsets(int lane) {
  NatOff<D> n;
  const int row = lane & 31, g = lane >> 5;
#pragma unroll
  for (int st = 0; st < D / 16; ++st) n.off[st] = tile_off<D>(row, 2 * st + g);
  return n;
}
template <int D>
__device__ __forceinline__ bf16x8 frag_nat(const char* tile, const NatOff<D>& n, int row_block, int step) {
  return *reinterpret_cast<const bf16x8*>(tile + n.off[step] + row_block * 32 * (2 * D));
}

// Transposed fragment (ds_read_b64_tr_b16): lane <-> column (d0 + l%32) of the tile, the 8
// values run over tile rows {r0 + 4g + 0..3, r0 + 8 + 4g + 0..3}, r0 a multiple of 16.
// Within each group of 16 lanes the instruction returns to lane i element (i%4) of the 8-byte
// row segments addressed by lanes 4j + i/4 (j = 0..3): lane i supplies the address of row
// (i/4), column segment 4*(i%4) of its group's 16 columns.
// TrOff holds the per-lane byte offsets for r0 = 0 of both 4-row halves and every 32-column block.
template <int D>
struct TrOff {
  int lo[D / 32], hi[D / 32];
};
template <int D>
__device__ __forceinline__ TrOff<D> tr_offsets(int lane) {
  TrOff<D> t;
  const int row_a = 4 * (lane >> 5) + ((lane & 15) >> 2);  // 4g + (l%16)/4
  const int row_b = row_a + 8;
  const int col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    const int c = db * 32 + col;
    t.lo[db] = tile_off<D>(row_a, c >> 3) + ((c & 7) << 1);
    t.hi[db] = tile_off<D>(row_b, c >> 3) + ((c & 7) << 1);
  }
  return t;
}
template <int D>
__device__ __forceinline__ bf16x8 frag_tr(const char* tile, const TrOff<D>& t, int r0, int db) {
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PEAGLE_LDS_PTR(s16x4, tile + t.lo[db] + r0 * (2 * D)));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PEAGLE_LDS_PTR(s16x4, tile + t.hi[db] + r0 * (2 * D)));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// Asynchronous global -> LDS copies.  dma16_untracked: 16 bytes per lane (global_load_lds_dwordx4), lane
// l's bytes land at lds_addr + 16*l, so one call fills 1 KiB of LDS per wave; dma4_untracked: 4 bytes per
// lane (global_load_lds_dword), lane l's dword lands at lds_addr + 4*l.  lds_addr is a scalar:
// lds_scalar_addr() of a wave-uniform pointer, plus wave-uniform offsets (so that no vector instruction
// is spent on it).  Completion is counted by vmcnt of the issuing wave only: dma_publish() makes the
// data visible to the other waves.
//
// The instruction is issued through an assembly statement rather than the compiler's builtin, hence
// "untracked".  The compiler counts a copy made with the builtin as an outstanding memory access of
// unknown LDS destination and makes the wave wait for ALL of them before its next LDS read, whichever
// buffer that read touches (and before every workgroup barrier with its fence); a kernel that issues the
// next tile's copy and then computes on the current one so stalls for the copy's whole latency unless
// another workgroup fills the gap.  Issued this way the copy is invisible to that bookkeeping (the
// hardware counter still counts it, so the compiler's own waits can only become longer, never too
// short), and the caller alone orders it: nothing may read or overwrite the destination before
// dma_publish() / wait_outstanding().  M0 carries the LDS address, as it would for the builtin; it is
// declared clobbered, and no kernel here mixes the two forms.
__device__ __forceinline__ uint32_t lds_scalar_addr(const char* lds_ptr) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)PEAGLE_LDS_PTR(char, lds_ptr));
}
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // "clobber list contains reserved registers: m0": intended, see above
__device__ __forceinline__ void dma16_untracked(const void* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gsrc), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void dma4_untracked(const void* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(gsrc), "s"(lds_addr) : "memory", "m0");
}
// The same copies with the global address split into a wave-uniform base (scalar registers) and a 32-bit
// per-lane byte offset: when the offsets of a lane do not change from tile to tile, a copy costs no vector
// instruction at all.  The offset is unsigned: the addressed range must lie within 4 GiB of the base.
__device__ __forceinline__ void dma16_untracked(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(sbase), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void dma4_untracked(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" : : "v"(voff), "s"(sbase), "s"(lds_addr) : "memory", "m0");
}
// A pointer the compiler can prove wave-uniform (so that it lives in scalar registers).
template <class T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
  const uint64_t u = (uint64_t)(uintptr_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return reinterpret_cast<const T*>((uintptr_t)(((uint64_t)hi << 32) | lo));
}
#pragma clang diagnostic pop

// Wait until every global -> LDS copy this wave has issued has landed (vmcnt(0)), then
// synchronise the workgroup: after it, all waves may read what any wave copied, and the buffers
// read before it may be overwritten.  The wait is explicit because a workgroup barrier by itself
// only orders ordinary LDS traffic; it is an assembly statement with a memory clobber so that it
// stays behind every earlier LDS read.
__device__ __forceinline__ void dma_publish() {
  asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
  __syncthreads();
}

// Wait until at most N of this wave's vector-memory accesses are outstanding (they complete in issue
// order, so this waits for all but the N youngest).  Like dma_publish() it is an assembly statement with a
// memory clobber: nothing moves across it.
template <int N>
__device__ __forceinline__ void wait_outstanding() {
  static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
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

// v_permlane32_swap exchanges the upper half of its first operand with the lower half of the
// second: with both set to x, the first result holds x[lane%32] in every lane and the second
// x[32 + lane%32].
// (Vector elements are copied to scalars before any __builtin_bit_cast: applied directly to an
// element expression such as r[1], the cast reads element 0 with this compiler.)
__device__ __forceinline__ void swap_halves(float x, float& lo, float& hi) {
  typedef __attribute__((ext_vector_type(2))) uint32_t u2;
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const u2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t a = r[0], b = r[1];
  lo = __builtin_bit_cast(float, a);
  hi = __builtin_bit_cast(float, b);
}
// max / sum over the two lanes (l, l^32) that share an MFMA column
__device__ __forceinline__ float max_halves(float x) {
  float lo, hi;
  swap_halves(x, lo, hi);
  return __builtin_fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_halves(float x) {
  float lo, hi;
  swap_halves(x, lo, hi);
  return lo + hi;
}

// acc + lo + hi of one packed bf16 pair, accumulated in fp32 (v_dot2_f32_bf16 against ones)
__device__ __forceinline__ float add_pair_bf16(uint32_t pair, float acc) {
  const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), ones, acc, false);
}

// 8 consecutive C registers (one 16-wide contraction step) -> bf16x8 B operand; also adds the
// eight rounded values to `sum`.
__device__ __forceinline__ bf16x8 pack8_sum(const f32x16& x, int t, float& sum) {
  u32x4 u;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    u[i] = pack_bf16(x[8 * t + 2 * i], x[8 * t + 2 * i + 1]);
    sum = add_pair_bf16(u[i], sum);
  }
  return __builtin_bit_cast(bf16x8, u);
}

}  // namespace peagle
