// Rotary position embedding of the drafter's attention (Sec. 2 of the paper: a LLaMA 3 style decoder
// with RoPE): device helpers shared by the rotation kernels and by the gradient epilogues of the
// attention kernels.
//
// The stored token (anchor i, depth d) stands at sequence position p = i + d, because depth d predicts
// the token d+1 ahead of its anchor (Sec. 3).  Feature pair (j, j + D/2) of a head vector turns by the
// angle p * base^(-2j/D); the table holds, per position, D/2 cosines followed by D/2 sines (fp32).
#pragma once

#include "mfma_util.h"
#include "tilemap.h"

namespace peagle {

// Sequence position of a stored token.  Dense maps: token t = d*L + i.  Sampled / packed maps list it.
__device__ __forceinline__ int token_position(const DeviceTileMap& tm, int tok, int L) {
  if (tm.tok_posid) return tm.tok_posid[tok];
  const int d = tok / L;
  return tok - d * L + d;
}

// Four feature pairs at once: lo = features [d0, d0+4), hi = features [D/2 + d0, D/2 + d0 + 4),
// cs / sn their cosines and sines.  Forward: (lo, hi) <- (lo cos - hi sin, hi cos + lo sin);
// the inverse (= transpose, which gradients take) flips the sign of the sines.
template <bool INVERSE>
__device__ __forceinline__ void rope_turn4(f32x4& lo, f32x4& hi, const f32x4 cs, const f32x4 sn) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float s = INVERSE ? -sn[j] : sn[j];
    const float a = lo[j], b = hi[j];
    lo[j] = __builtin_fmaf(a, cs[j], -(b * s));
    hi[j] = __builtin_fmaf(b, cs[j], a * s);
  }
}

}  // namespace peagle
