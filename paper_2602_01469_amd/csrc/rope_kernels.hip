// Rotary position embedding around the attention step (Sec. 2 of the paper; position ids
// p = anchor + depth from Sec. 3): the table of angles, and the rotation of a [T, H, D] bf16 tensor.
// Both are pure streaming work (HBM bound); the counter-rotation of dQ and dK happens in the
// epilogues of the attention kernels, on the fp32 values before they are stored.
#include "attn_kernels.h"
#include "rope_util.h"

namespace peagle {

namespace {

// table[p][0][j] = cos(p * base^(-2j/D)), table[p][1][j] = sin(...), j < D/2.  Angles reach tens of
// thousands of radians, so they are formed and reduced in double precision.
__global__ __launch_bounds__(256) void rope_table_kernel(double log_base, int D, int n_pos, float* table) {
  const int half = D / 2;
  const size_t n = (size_t)n_pos * half;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
    const int p = (int)(idx / half), j = (int)(idx % half);
    const double theta = exp(-(2.0 * j / D) * log_base);
    double s, c;
    sincos((double)p * theta, &s, &c);
    table[(size_t)p * D + j] = (float)c;
    table[(size_t)p * D + half + j] = (float)s;
  }
}

// One thread per (token, head, 8 features of the lower half): reads the 8 features and their 8
// partners of the upper half (16 bytes each), turns the 8 pairs in fp32, rounds once to bf16.
template <int D, bool INVERSE>
__global__ __launch_bounds__(256) void rope_rotate_kernel(const __bf16* x, __bf16* out, int H, int T, DeviceTileMap tm,
                                                          int L, const float* table) {
  constexpr int kChunks = D / 16;
  const size_t n = (size_t)T * H * kChunks;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % kChunks);
    const size_t th = idx / kChunks;  // token * H + head
    const int tok = (int)(th / H);
    const float* row = table + (size_t)token_position(tm, tok, L) * D + c * 8;
    const __bf16* src = x + th * D + c * 8;
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(src);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(src + D / 2);
    u32x4 wa, wb;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      f32x4 lo, hi;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lo[j] = (float)a[4 * q + j];
        hi[j] = (float)b[4 * q + j];
      }
      rope_turn4<INVERSE>(lo, hi, *reinterpret_cast<const f32x4*>(row + 4 * q),
                          *reinterpret_cast<const f32x4*>(row + D / 2 + 4 * q));
      wa[2 * q] = pack_bf16(lo[0], lo[1]);
      wa[2 * q + 1] = pack_bf16(lo[2], lo[3]);
      wb[2 * q] = pack_bf16(hi[0], hi[1]);
      wb[2 * q + 1] = pack_bf16(hi[2], hi[3]);
    }
    __bf16* dst = out + th * D + c * 8;
    *reinterpret_cast<u32x4*>(dst) = wa;
    *reinterpret_cast<u32x4*>(dst + D / 2) = wb;
  }
}

// First drafter layer (Sec. 2: every multi-token position is fed the shared hidden state and the mask-token
// embedding): tokens [0, L0) - the depth-0 positions - have rows of their own in x0 [L0, H, D], every later
// token reads the one vector x_shared [H, D].  ROTATE: turn each row by its token's position (keys);
// otherwise plain copies (values).
template <int D, bool ROTATE>
__global__ __launch_bounds__(256) void expand_shared_kernel(const __bf16* x0, const __bf16* x_shared, __bf16* out, int H,
                                                            int T, int L0, DeviceTileMap tm, int L, const float* table) {
  constexpr int kChunks = D / 16;
  const size_t n = (size_t)T * H * kChunks;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % kChunks);
    const size_t th = idx / kChunks;  // token * H + head
    const int tok = (int)(th / H), h = (int)(th - (size_t)tok * H);
    const __bf16* src = (tok < L0 ? x0 + th * D : x_shared + (size_t)h * D) + c * 8;
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(src);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(src + D / 2);
    __bf16* dst = out + th * D + c * 8;
    if (!ROTATE) {
      *reinterpret_cast<bf16x8*>(dst) = a;
      *reinterpret_cast<bf16x8*>(dst + D / 2) = b;
      continue;
    }
    const float* row = table + (size_t)token_position(tm, tok, L) * D + c * 8;
    u32x4 wa, wb;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      f32x4 lo, hi;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lo[j] = (float)a[4 * q + j];
        hi[j] = (float)b[4 * q + j];
      }
      rope_turn4<false>(lo, hi, *reinterpret_cast<const f32x4*>(row + 4 * q),
                        *reinterpret_cast<const f32x4*>(row + D / 2 + 4 * q));
      wa[2 * q] = pack_bf16(lo[0], lo[1]);
      wa[2 * q + 1] = pack_bf16(lo[2], lo[3]);
      wb[2 * q] = pack_bf16(hi[0], hi[1]);
      wb[2 * q + 1] = pack_bf16(hi[2], hi[3]);
    }
    *reinterpret_cast<u32x4*>(dst) = wa;
    *reinterpret_cast<u32x4*>(dst + D / 2) = wb;
  }
}

// Gradients of the shared vectors: column sums of acc [T][cols] (fp32; the per-wave sums of the chain keys' dK or
// dV that the dK/dV kernel leaves - a few thousand rows).  A block of 256 threads is 16 row lanes x 16 column
// pieces of 16 bytes: row lane r adds up rows r, r + 16, ... of its piece, eight loads in flight, and the 16 lanes
// are then summed through LDS in a fixed order (deterministic).  gridDim.y selects dK or dV.
__global__ __launch_bounds__(256) void shared_grad_reduce(const float* acc_k, const float* acc_v, float* out_k,
                                                          float* out_v, int T, int cols) {
  __shared__ f32x4 red[256];
  const float* acc = blockIdx.y ? acc_v : acc_k;
  float* out = blockIdx.y ? out_v : out_k;
  const int c4 = blockIdx.x * 16 + (threadIdx.x & 15), rl = threadIdx.x >> 4, n4 = cols / 4;
  f32x4 sum = {0.f, 0.f, 0.f, 0.f};
  if (c4 < n4) {
    const float* col = acc + c4 * 4;
    int t = rl;
    for (; t + 7 * 16 < T; t += 8 * 16) {
      f32x4 x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) x[u] = *reinterpret_cast<const f32x4*>(col + (size_t)(t + 16 * u) * cols);
      sum += ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
    }
    for (; t < T; t += 16) sum += *reinterpret_cast<const f32x4*>(col + (size_t)t * cols);
  }
  red[threadIdx.x] = sum;
  __syncthreads();
  if (rl == 0 && c4 < n4) {
    for (int l = 1; l < 16; ++l) sum += red[threadIdx.x + 16 * l];
    *reinterpret_cast<f32x4*>(out + c4 * 4) = sum;
  }
}

inline unsigned grid_for(size_t n) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  return (unsigned)(blocks ? blocks : 1);
}

}  // namespace

hipError_t launch_rope_table(double base, int D, int n_pos, float* table, hipStream_t stream) {
  const size_t n = (size_t)n_pos * (D / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3(grid_for(n)), dim3(256), 0, stream, log(base), D, n_pos, table);
  return hipGetLastError();
}

hipError_t launch_rope_rotate(const void* x, void* out, int H, int T, int D, const DeviceTileMap& tm, int L,
                              const float* table, bool inverse, hipStream_t stream, KernelTimer* timer) {
  const size_t n = (size_t)T * H * (D / 16);
  if (n == 0) return hipSuccess;
  const dim3 grid(grid_for(n)), block(256);
  const __bf16* xi = (const __bf16*)x;
  __bf16* xo = (__bf16*)out;
  hipError_t begin = timer ? timer->begin(kKindRope, stream) : hipSuccess;
  if (D == 64) {
    if (inverse) hipLaunchKernelGGL((rope_rotate_kernel<64, true>), grid, block, 0, stream, xi, xo, H, T, tm, L, table);
    else hipLaunchKernelGGL((rope_rotate_kernel<64, false>), grid, block, 0, stream, xi, xo, H, T, tm, L, table);
  } else {
    if (inverse) hipLaunchKernelGGL((rope_rotate_kernel<128, true>), grid, block, 0, stream, xi, xo, H, T, tm, L, table);
    else hipLaunchKernelGGL((rope_rotate_kernel<128, false>), grid, block, 0, stream, xi, xo, H, T, tm, L, table);
  }
  hipError_t e = hipGetLastError();
  if (timer && begin == hipSuccess) begin = timer->end(stream);
  return e != hipSuccess ? e : begin;
}

hipError_t launch_expand_shared(const void* x0, const void* x_shared, void* out, int H, int T, int L0, int D,
                                const DeviceTileMap& tm, int L, const float* table, hipStream_t stream) {
  const size_t n = (size_t)T * H * (D / 16);
  if (n == 0) return hipSuccess;
  const dim3 grid(grid_for(n)), block(256);
  const __bf16 *a = (const __bf16*)x0, *b = (const __bf16*)x_shared;
  __bf16* o = (__bf16*)out;
  if (D == 64) {
    if (table) hipLaunchKernelGGL((expand_shared_kernel<64, true>), grid, block, 0, stream, a, b, o, H, T, L0, tm, L, table);
    else hipLaunchKernelGGL((expand_shared_kernel<64, false>), grid, block, 0, stream, a, b, o, H, T, L0, tm, L, table);
  } else {
    if (table) hipLaunchKernelGGL((expand_shared_kernel<128, true>), grid, block, 0, stream, a, b, o, H, T, L0, tm, L, table);
    else hipLaunchKernelGGL((expand_shared_kernel<128, false>), grid, block, 0, stream, a, b, o, H, T, L0, tm, L, table);
  }
  return hipGetLastError();
}

hipError_t launch_shared_grads(const float* part_k, const float* part_v, int rows, float* dk_shared, float* dv_shared,
                               int cols, hipStream_t stream) {
  hipLaunchKernelGGL(shared_grad_reduce, dim3((unsigned)((cols / 4 + 15) / 16), 2), dim3(256), 0, stream, part_k, part_v,
                     dk_shared, dv_shared, rows, cols);
  return hipGetLastError();
}

}  // namespace peagle
