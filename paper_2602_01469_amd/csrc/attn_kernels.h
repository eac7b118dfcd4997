// Kernel parameter blocks and host launchers of the attention path.
#pragma once

#include <hip/hip_runtime.h>

#include <vector>

#include "tilemap.h"

namespace peagle {

struct FwdParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  __bf16* o;
  float* lse;          // [Hq, T]
  DeviceTileMap tm;
  int L, T, Hq, Hkv;
  int rt_lo, rt_hi;    // row tiles of the segment
  float c_log2;        // softmax scale * log2(e)
  const __bf16* v_shared;  // null, or [Hkv, D]: the value row of every chain key (first-layer form; v then holds
                           // the depth-0 rows only)
};

struct BwdParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const __bf16* o;
  const __bf16* d_o;
  const float* lse;    // [Hq, T]
  __bf16* dq;
  float* dk_acc;       // [T, Hkv, D]
  float* dv_acc;
  float* delta;        // workspace [Hq, T]: -rowsum(dO * O), written by the dQ kernel
  float* nlse;         // workspace [Hq, T]: -lse / scale, written by the dQ kernel
  float* dk_part;      // workspace [Hq, L64, D]: per-query-head dK of the depth-0 keys
  float* dv_part;
  DeviceTileMap tm;
  int L, T, Hq, Hkv, L64;
  int rt_lo, rt_hi;
  int s_lo, s_hi, cropped;  // segment boundary indices of the row range; cropped: rt_hi cuts the last segment short
  int n_d0_items;       // filled by the launcher: depth-0 work items (key-tile pairs x query heads)
  int n_d0_tiles;       // filled by the launcher: depth-0 key tiles visible to the segment are [d0_tile_lo, n_d0_tiles)
  int d0_tile_lo;
  int clip_rows;        // filled by the launcher: [rt_lo, rt_hi) covers only part of the segments s_lo..s_hi
  int d0_split, d0_step;  // filled by the launcher: depth-0 pairs are dealt in passes, [0, d0_split) then d0_step at a time
  int fast_rows;        // Q-shaped tensors and the [Hq, T] statistics span less than 4 GiB: row copies may use 32-bit offsets
  int chain_accumulate; // chain keys: add to dk_acc/dv_acc instead of overwriting
  float c_log2, scale;
  const float* rope_table;  // null, or [positions][2][D/2] cosines and sines: q and k are rotated copies, and dQ / dK
                            // are turned back to the unrotated inputs' frame before they are stored
  // First-layer form (every chain key carries the same K and V vector, rotated by its position): v_shared [Hkv, D]
  // is the value row of every chain key (v then holds the depth-0 rows only), and the chain keys' dK / dV are not
  // stored per key but summed over the 32 keys of a wave into shared_dk_part / shared_dv_part
  // [(row tile * chain-tile pairs + pair) * 4 + wave][Hkv][D], which a reduction then adds up.  All null otherwise.
  const __bf16* v_shared;
  float* shared_dk_part;
  float* shared_dv_part;
};

// Inference-side drafting step (Sec. 2 of the paper: all K draft positions in one forward pass): the K
// rows of each request against its paged KV cache plus the K new keys.
struct DecodeParams {
  const __bf16* q_new;         // [C, K, Hq, D]
  const __bf16* k_new;         // [C, K, Hkv, D]
  const __bf16* v_new;
  const __bf16* k_pages;       // [n_pages, Hkv, 64, D]
  const __bf16* v_pages;
  const int32_t* block_table;  // [C, max_pages] page of each 64-token block of a request's context
  const int32_t* ctx_len;      // [C] cached tokens per request
  __bf16* o;                   // [C, K, Hq, D]
  float* lse;                  // [C, Hq, K]
  int32_t* status;             // [C] or null: 1 if the request's block table or length was out of range
  float* part_o;               // workspace [C, Hkv, n_splits, rows_pad, D]: unnormalised partial outputs
  float* part_ml;              // workspace [C, Hkv, n_splits, 3, rows_pad]: reference max (log2), row sum, flag
  int C, K, Hq, Hkv, n_pages, max_pages, n_splits, rows_pad;
  float c_log2;
};
hipError_t launch_draft_decode(const DecodeParams& p, int D, hipStream_t stream);

// Optional per-kernel timing: an event pair is recorded around every launch on the launch stream.
enum KernelKind { kKindFwd = 0, kKindDq = 1, kKindDkDv = 2, kKindReduce = 3, kKindRope = 4, kNumKinds = 5 };
struct KernelTimer {
  struct Span { hipEvent_t start, stop; int kind; };
  std::vector<Span> spans;
  hipError_t begin(int kind, hipStream_t stream);
  hipError_t end(hipStream_t stream);
  // Waits for the recorded work, adds the elapsed ms per kind into ms[] / launches[], frees the events.
  hipError_t collect(float* ms, int32_t* launches);
  ~KernelTimer();
};

hipError_t launch_fwd(const FwdParams& p, int D, hipStream_t stream, KernelTimer* timer = nullptr);
// a_hi: end anchor of the segment (depth-0 keys [0, a_hi) are visible); depth-0 keys with anchor
// below acc_below are added to dk_acc/dv_acc, the others overwritten.
hipError_t launch_bwd(const BwdParams& p, int D, int key_lo, int a_hi, int acc_below, hipStream_t stream,
                      KernelTimer* timer = nullptr);
// Dense bf16 MFMA issue loop on every CU: the measured matrix-core ceiling of the device, in TFLOP/s, on
// constant small-integer operands or on changing pseudo-random ones (the chip clocks lower under the latter).
hipError_t measure_mfma_ceiling(hipStream_t stream, bool random_operands, float* tflops);
hipError_t launch_cast_bf16(const float* src, void* dst_bf16, size_t n, hipStream_t stream);
// Rotary embedding: table [n_pos][2][D/2] of cosines and sines; rotation of a bf16 [T, H, D] tensor
// by each token's position (inverse: the transpose).
hipError_t launch_rope_table(double base, int D, int n_pos, float* table, hipStream_t stream);
// First-layer form: expansion of (own depth-0 rows, one shared vector for every later token) into a full
// [T, H, D] tensor, rotated when a table is given.
hipError_t launch_expand_shared(const void* x0, const void* x_shared, void* out, int H, int T, int L0, int D,
                                const DeviceTileMap& tm, int L, const float* table_or_null, hipStream_t stream);
// Column sums of part_k / part_v [rows][cols] (the per-wave sums of the chain keys' gradients) into
// dk_shared / dv_shared [cols], in a fixed order.
hipError_t launch_shared_grads(const float* part_k, const float* part_v, int rows, float* dk_shared, float* dv_shared,
                               int cols, hipStream_t stream);
hipError_t launch_rope_rotate(const void* x, void* out, int H, int T, int D, const DeviceTileMap& tm, int L,
                              const float* table, bool inverse, hipStream_t stream, KernelTimer* timer = nullptr);

}  // namespace peagle
