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

// Gradients of the shared vectors: column sums of the chain tokens' rows [L0, T) of acc [T, cols] (fp32),
// in two deterministic stages.  Stage 1: block b sums the tokens L0 + b, L0 + b + nblk, ... into
// partial[b][cols]; stage 2 sums the partials, a thread per 16-byte column piece.  Stage 1 also copies the
// depth-0 rows [0, L0) to their own output (all blocks).  gridDim.y selects dK or dV.
__global__ __launch_bounds__(256) void shared_grad_stage1(const float* acc_k, const float* acc_v, float* partial,
                                                          float* out0_k, float* out0_v, int T, int L0, int cols) {
  __shared__ f32x4 red[256];
  const float* acc = blockIdx.y ? acc_v : acc_k;
  float* out0 = blockIdx.y ? out0_v : out0_k;
  const int nblk = gridDim.x, b = blockIdx.x, n4 = cols / 4;
  // Threads are laid out as (token lane, 16-byte column piece): consecutive threads read consecutive pieces of
  // one row, `lanes` rows at a time, four rows in flight per thread; the token lanes of a piece are then summed
  // through LDS in a fixed order.
  const int lanes = n4 <= 256 ? 256 / n4 : 1;
  const int tl = n4 <= 256 ? threadIdx.x / n4 : 0;
  for (int c0 = 0; c0 < n4; c0 += 256) {
    const int c4 = c0 + (n4 <= 256 ? threadIdx.x % n4 : threadIdx.x);
    const bool on = c4 < n4 && tl < lanes;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    if (on) {
      const size_t stride = (size_t)nblk * lanes;
      size_t t = (size_t)L0 + b + (size_t)tl * nblk;
      for (; t + 3 * stride < (size_t)T; t += 4 * stride) {
        const f32x4 x0 = *reinterpret_cast<const f32x4*>(acc + t * cols + c4 * 4);
        const f32x4 x1 = *reinterpret_cast<const f32x4*>(acc + (t + stride) * cols + c4 * 4);
        const f32x4 x2 = *reinterpret_cast<const f32x4*>(acc + (t + 2 * stride) * cols + c4 * 4);
        const f32x4 x3 = *reinterpret_cast<const f32x4*>(acc + (t + 3 * stride) * cols + c4 * 4);
        sum += (x0 + x1) + (x2 + x3);
      }
      for (; t < (size_t)T; t += stride) sum += *reinterpret_cast<const f32x4*>(acc + t * cols + c4 * 4);
      for (size_t t0 = (size_t)b + (size_t)tl * nblk; t0 < (size_t)L0; t0 += stride)
        *reinterpret_cast<f32x4*>(out0 + t0 * cols + c4 * 4) = *reinterpret_cast<const f32x4*>(acc + t0 * cols + c4 * 4);
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    if (on && tl == 0) {
      for (int l = 1; l < lanes; ++l) sum += red[threadIdx.x + l * n4];
      *reinterpret_cast<f32x4*>(partial + ((size_t)blockIdx.y * nblk + b) * cols + c4 * 4) = sum;
    }
    __syncthreads();
  }
}
__global__ __launch_bounds__(256) void shared_grad_stage2(const float* partial, float* out_k, float* out_v, int nblk,
                                                          int cols) {
  float* out = blockIdx.y ? out_v : out_k;
  const int c4 = blockIdx.x * blockDim.x + threadIdx.x;  // one thread per 16-byte column piece
  if (c4 >= cols / 4) return;
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, s2 = s0, s3 = s0;
  const float* src = partial + (size_t)blockIdx.y * nblk * cols + c4 * 4;
  int b = 0;
  for (; b + 3 < nblk; b += 4) {
    s0 += *reinterpret_cast<const f32x4*>(src + (size_t)b * cols);
    s1 += *reinterpret_cast<const f32x4*>(src + (size_t)(b + 1) * cols);
    s2 += *reinterpret_cast<const f32x4*>(src + (size_t)(b + 2) * cols);
    s3 += *reinterpret_cast<const f32x4*>(src + (size_t)(b + 3) * cols);
  }
  for (; b < nblk; ++b) s0 += *reinterpret_cast<const f32x4*>(src + (size_t)b * cols);
  *reinterpret_cast<f32x4*>(out + c4 * 4) = (s0 + s1) + (s2 + s3);
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

hipError_t launch_shared_grads(const float* acc_k, const float* acc_v, float* partial, int n_partial_blocks, float* dk0,
                               float* dv0, float* dk_shared, float* dv_shared, int T, int L0, int cols,
                               hipStream_t stream) {
  hipLaunchKernelGGL(shared_grad_stage1, dim3((unsigned)n_partial_blocks, 2), dim3(256), 0, stream, acc_k, acc_v, partial,
                     dk0, dv0, T, L0, cols);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(shared_grad_stage2, dim3((unsigned)((cols / 4 + 63) / 64), 2), dim3(64), 0, stream, partial,
                     dk_shared, dv_shared, n_partial_blocks, cols);
  return hipGetLastError();
}

}  // namespace peagle
