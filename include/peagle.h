/*
 * peagle.h - C ABI of the MI355X (gfx950) parallel-drafting attention path of P-EAGLE.
 *
 * The library computes, for the training of the P-EAGLE drafter, masked attention over the
 * expanded sequence of Sec. 3 of the paper: a sequence of L tokens becomes T = L*K positions,
 * one per (anchor i in [0,L), prediction depth d in [0,K)); depth 0 is the ordinary next-token
 * position, depths 1..K-1 carry the shared hidden state.  The parallel-prediction mask
 * (Sec. 3, PARD paragraph: a depth-d row sees depths <= d only; Sec. 3.2, Challenge 2:
 * position p at depth d depends on position p-1 at depth d-1) reads, in anchor coordinates:
 *
 *     row (i,d) sees key (j,e)   iff   (e == 0 and j <= i)  or  (j == i and 1 <= e <= d).
 *
 * Storage order of every [T, ...] tensor is depth-major: t = d*L + i (the G0|G1|... blocks of
 * Fig. 3).  Query head h uses KV head h / (Hq/Hkv).
 *
 * Conventions shared by all entry points
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library never frees or keeps caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All GPU work is
 *     enqueued on it; no entry point synchronises the device except peagle_build_tilemap
 *     (whose upload is complete on return).
 *   - Return value: PEAGLE_OK (0) or a negative peagle_status.  Arguments are validated on the
 *     host before anything is launched, so every error path can be exercised without a GPU.
 *     Nothing is printed, thrown or aborted.
 */
#ifndef PEAGLE_H
#define PEAGLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum peagle_status {
  PEAGLE_OK = 0,
  PEAGLE_EINVAL = -1,       /* bad scalar argument (negative size, Hq % Hkv != 0, seg out of range ...) */
  PEAGLE_ENULL = -2,        /* a required pointer is NULL */
  PEAGLE_ESHAPE = -3,       /* shape does not fit the tile map (L > L_max, K mismatch) */
  PEAGLE_EBOUNDS = -4,      /* segment bounds not strictly increasing from 0 to L_max, or an inner bound
                               is not a multiple of the anchors-per-row-tile */
  PEAGLE_EUNSUPPORTED = -5, /* head_dim not in {64, 128}, K > 128, unknown layout */
  PEAGLE_EWORKSPACE = -6,   /* workspace missing or smaller than peagle_workspace_bytes() */
  PEAGLE_EHIP = -7,         /* a HIP runtime call failed (allocation, copy, launch) */
  PEAGLE_ENODEVICE = -8     /* the tile map was built host-only (device < 0) and cannot be used to launch */
} peagle_status;

#define PEAGLE_LAYOUT_DEPTH_MAJOR 0   /* t = d*L + i; the only layout */

/* Problem shape of one call.  L may be any value in [1, L_max of the tile map]: the shorter
 * sequence uses the prefix of the tile map (position invariance of the mask, Sec. 3.1). */
typedef struct peagle_shape {
  int32_t L;       /* anchor tokens */
  int32_t K;       /* prediction depths; must equal the tile map's K */
  int32_t Hq;      /* query heads */
  int32_t Hkv;     /* key/value heads, divides Hq */
  int32_t D;       /* head dimension, 64 or 128 */
  int32_t layout;  /* PEAGLE_LAYOUT_DEPTH_MAJOR */
  float scale;     /* softmax scale applied to q.k (e.g. 1/sqrt(D)) */
} peagle_shape_t;

/* Opaque tile map: library-owned host copy plus (unless built host-only) a device copy. */
typedef struct peagle_tilemap peagle_tilemap_t;

/* Tile classes of peagle_tilemap_classes(). */
#define PEAGLE_TILE_EMPTY 0
#define PEAGLE_TILE_FULL 1
#define PEAGLE_TILE_PARTIAL 2

typedef struct peagle_tilemap_info {
  int32_t L_max, K, S;
  int32_t anchors_per_row_tile;  /* A = 128 / K (integer division): a row tile is A anchors x all K depths */
  int32_t rows_per_tile;         /* 128 (A*K of them in use) */
  int32_t keys_per_tile;         /* 64 */
  int32_t n_row_tiles;           /* ceil(L_max / A) */
  int32_t n_depth0_key_tiles;    /* ceil(L_max / 64): key tile c holds depth-0 anchors [64c, 64c+64) */
  int32_t n_chain_sub_tiles;     /* ceil(A*(K-1) / 64): chain key tiles per row tile */
  int32_t n_key_tiles;           /* depth-0 tiles followed by n_row_tiles * n_chain_sub_tiles chain tiles */
  int64_t n_full;                /* non-empty tile pairs whose every element is visible */
  int64_t n_partial;             /* tile pairs that need a bitmask */
  int32_t n_masks;               /* distinct bitmasks in the pool (128 rows x 64 bits each) */
  int64_t device_bytes;          /* bytes of the device copy (0 if host-only) */
  int64_t tokens;                /* stored tokens of a length-L_max sequence */
  int32_t sampled;               /* 1 if built by peagle_build_tilemap_sampled */
} peagle_tilemap_info_t;

/*
 * Mask -> tile map, built once for the maximum length (amortized mask construction, Sec. 3.1)
 * with the segment boundaries of sequence partitioning (Sec. 3.2, boundaries B of Algorithm 1,
 * given explicitly because L/S need not be an integer).
 *
 *   L_max       maximum anchor count, >= 1
 *   K           prediction depths, 1..128
 *   seg_bounds  host, int32[S+1], anchor indices, seg_bounds[0] = 0 < ... < seg_bounds[S] = L_max;
 *               every inner bound must be a multiple of A = 128/K.  NULL with S = 1 means {0, L_max}.
 *   device      HIP device ordinal for the device copy, or -1 for a host-only map (introspection only)
 *   out         receives the handle; release with peagle_tilemap_destroy
 *
 * Geometry: a row tile is A consecutive anchors at all K depths (row r of the tile is depth r/A,
 * anchor r%A).  Its keys come from two streams: depth-0 key tiles of 64 consecutive anchors, and
 * the chain key tiles holding the depth >= 1 positions of the tile's own anchors (key k of the
 * chain stream is depth 1 + k/A, anchor k%A).  Each (row tile, key tile) pair is classified
 * empty / full / partial from interval tests; partial pairs point into a pool of de-duplicated
 * bitmasks (the pool has O(1) entries because the mask is position-invariant).
 */
int peagle_build_tilemap(int32_t L_max, int32_t K, const int32_t* seg_bounds, int32_t S, int32_t device,
                         peagle_tilemap_t** out);

void peagle_tilemap_destroy(peagle_tilemap_t* tm);

int peagle_tilemap_info(const peagle_tilemap_t* tm, peagle_tilemap_info_t* info /* host, out */);

/*
 * Host-side expansion of the tile map back to the element mask, for bit-exact checks.
 * For the query rows t in [row_begin, row_end) (token indices of a length-L problem, L <= L_max)
 * writes (row_end-row_begin) * ceil(T/8) bytes to bits_out (host), T = peagle_tilemap_tokens(tm, L):
 * bit (c % 8) of byte c/8 of a row is 1 iff key token c is visible.  With seg >= 0, rows outside
 * segment `seg` come out all zero.
 */
int peagle_tilemap_expand_rows(const peagle_tilemap_t* tm, int32_t L, int32_t seg, int64_t row_begin,
                               int64_t row_end, uint8_t* bits_out);

/* Dense class map: classes_out (host) receives n_row_tiles * n_key_tiles bytes, row-tile major,
 * each PEAGLE_TILE_EMPTY / _FULL / _PARTIAL. */
int peagle_tilemap_classes(const peagle_tilemap_t* tm, uint8_t* classes_out);

/* Bytes of device scratch that peagle_attn_bwd / peagle_attn_step_partitioned need for this shape. */
size_t peagle_workspace_bytes(const peagle_tilemap_t* tm, const peagle_shape_t* shape);

/*
 * Attention forward over the query rows of one segment (seg in [0,S)) or of the whole sequence
 * (seg = -1): S = scale * Q K^T on non-empty tiles, mask bits on partial tiles, online softmax,
 * O = P V, LSE = ln sum exp (natural log, scale included).  The attention is the O((nK)^2) term
 * of Sec. 3; a segment's keys are the cumulative depth-0 context plus its own chains (Sec. 3.2).
 *
 *   q        device, bf16 [T, Hq, D]           k, v   device, bf16 [T, Hkv, D]
 *   o        device, bf16 [T, Hq, D]  (out; only the segment's rows are written)
 *   lse      device, fp32 [Hq, T]     (out; only the segment's rows are written)
 */
int peagle_attn_fwd(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg, const void* q,
                    const void* k, const void* v, void* o, float* lse, void* stream);

/*
 * Attention backward for the same rows: Delta = rowsum(dO * O), P = exp(S - LSE), dV = P^T dO,
 * dP = dO V^T, dS = P * (dP - Delta), dQ = scale * dS K, dK = scale * dS^T Q, with dK/dV summed
 * over the query heads of a KV group (each segment runs as a forward-backward pass of its own, Sec. 3.2).
 *
 *   o, d_o     device, bf16 [T, Hq, D]   (O from peagle_attn_fwd, upstream gradient)
 *   lse        device, fp32 [Hq, T]
 *   dq         device, bf16 [T, Hq, D]   (out; only the segment's rows are written)
 *   dk_acc     device, fp32 [T, Hkv, D]  (out; only keys visible to the segment are touched)
 *   dv_acc     device, fp32 [T, Hkv, D]
 *   accumulate 0: touched dK/dV elements are overwritten; 1: added to (caller zeroed or holds
 *              earlier segments' sums)
 *   workspace  device, >= peagle_workspace_bytes(); contents undefined before and after
 */
int peagle_attn_bwd(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg, const void* q,
                    const void* k, const void* v, const void* o, const void* d_o, const float* lse, void* dq,
                    float* dk_acc, float* dv_acc, int32_t accumulate, void* workspace, size_t ws_bytes,
                    void* stream);

/*
 * Within-sequence gradient accumulation (Sec. 3.2, Algorithm 1 for dense position sets): runs
 * forward + backward for segments seg_begin .. seg_end-1 one after another and accumulates dK/dV
 * across them in fp32.  Each query row is computed in exactly one segment.
 *
 * dK/dV need no zeroing when segments run in increasing order starting at 0: a depth-0 key first
 * touched by segment s is overwritten there and added to by later segments; chain keys are written
 * by their own segment only.  A call with seg_begin > 0 continues a run whose earlier segments
 * already ran on the same dk_acc/dv_acc.
 *
 *   dk_bf16, dv_bf16   device, bf16 [T, Hkv, D] or NULL: if given and seg_end == S, the fp32
 *                      sums are rounded once to bf16 into them after the last segment.
 */
int peagle_attn_step_partitioned(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg_begin,
                                 int32_t seg_end, const void* q, const void* k, const void* v, const void* d_o,
                                 void* o, float* lse, void* dq, float* dk_acc, float* dv_acc, void* dk_bf16,
                                 void* dv_bf16, void* workspace, size_t ws_bytes, void* stream);

/*
 * Tile map of a drop-token sampled sequence (Conditional Drop-token sampling, PARD paragraph of
 * Sec. 3: depth g keeps a geometrically shrinking subset of positions, n(1-r^K)/(1-r) in total,
 * Sec. 3.2).  A kept position p at depth g needs position p-1 at depth g-1 (Sec. 3.2,
 * Challenge 2), so per anchor the kept depths are a prefix: anchor i keeps depths
 * 0 .. depth_count[i]-1.
 *
 *   depth_count  host, int32[L], each in [1, K]
 *   seg_bounds   host, int32[S+1], 0 = b_0 < ... < b_S = L, any anchor indices (NULL with S = 1)
 *   assignment   which segment computes the rows of depth >= 1 (depth 0 always goes by position):
 *                PEAGLE_ASSIGN_BY_ANCHOR  - with their anchor, as in the dense map;
 *                PEAGLE_ASSIGN_ALGORITHM1 - as Algorithm 1 assigns them: depth 1 by its own position
 *                p = i+1, deeper depths inherit from (p-1, g-1), so the chain of anchor i is computed
 *                in the segment holding position i+1 (the last segment if i+1 is past the sequence).
 *                Outputs do not depend on the choice (every row is computed once, dK/dV are sums).
 *
 * Storage order of every [T, ...] tensor of such a sequence: depth-major, and within a depth the
 * anchors that keep it in ascending order; T = sum(depth_count) = peagle_tilemap_tokens(tm, L).
 * The map is built for this one sequence (the sample differs per example) and is used with
 * shape->L == L in every entry point that takes a tile map; all of them then index tensors of T
 * rows (lse is [Hq, T]).  Its row tiles are runs of consecutive anchors packed until their kept
 * positions fill 128 rows, so no matrix-core work is spent on dropped positions; the mask is the
 * dense parallel-prediction mask restricted to kept positions.  Segment s computes its rows
 * against the cumulative depth-0 context N_s = [0, b_{s+1}) and their own chains (Sec. 3.2).
 */
#define PEAGLE_ASSIGN_BY_ANCHOR 0
#define PEAGLE_ASSIGN_ALGORITHM1 1
int peagle_build_tilemap_sampled(const int32_t* depth_count, int32_t L, int32_t K, const int32_t* seg_bounds,
                                 int32_t S, int32_t assignment, int32_t device, peagle_tilemap_t** out);

/*
 * The general form of peagle_build_tilemap_sampled: a batch of n_seq sequences packed before the
 * n x K expansion of Sec. 3 (variable-length batches; the paper trains on sequences between a few
 * hundred and 20,000 tokens, Fig. 1), with or without drop-token sampling.
 *
 *   depth_count  host, int32[L] as above, or NULL: every anchor keeps all K depths (dense)
 *   L            total anchors of the batch
 *   seq_start    host, int32[n_seq+1], 0 = s_0 < ... < s_{n_seq} = L: sequence q owns the anchors
 *                [s_q, s_{q+1}); NULL with n_seq = 1 means one sequence
 *   seg_bounds   as above, over the anchors of the whole batch
 *
 * Anchors are numbered across the batch and storage is depth-major over the whole batch: block G0
 * holds every sequence's depth-0 positions, then G1, ... (the layout obtained by packing first and
 * expanding afterwards).  A row sees the depth-0 keys of its own sequence up to its anchor, and its
 * own chain; sequences do not see each other.  Row tiles never span two sequences.  Under
 * PEAGLE_ASSIGN_ALGORITHM1 a chain whose position i+1 is past its sequence stays in its anchor's
 * segment.
 */
int peagle_build_tilemap_packed(const int32_t* depth_count, int32_t L, int32_t K, const int32_t* seq_start,
                                int32_t n_seq, const int32_t* seg_bounds, int32_t S, int32_t assignment,
                                int32_t device, peagle_tilemap_t** out);

/*
 * Replaces the position set of a map made by peagle_build_tilemap_sampled / _packed, in place.
 * Drop-token samples change with every training example (Sec. 3, PARD paragraph); this keeps the
 * handle, its device allocation and its pinned staging buffer (they grow only when the new map
 * needs more room), so a training loop allocates nothing per step.  K stays that of the map;
 * the other arguments are those of peagle_build_tilemap_packed.
 *
 * The new map is copied to the device with one asynchronous copy on `stream` and is visible to
 * work enqueued on that stream after this call; work already enqueued on it keeps reading the old
 * map.  Work on other streams that still uses the map must have finished before the call.  The
 * call blocks only to wait for the previous rebuild's copy (the staging buffer is reused).
 * On error the map is unchanged if the arguments were rejected (EINVAL, ENULL, EBOUNDS,
 * EUNSUPPORTED: a dense map cannot be rebuilt) and unusable after PEAGLE_EHIP.
 */
int peagle_tilemap_rebuild(peagle_tilemap_t* tm, const int32_t* depth_count, int32_t L, const int32_t* seq_start,
                           int32_t n_seq, const int32_t* seg_bounds, int32_t S, int32_t assignment, void* stream);

/* Stored tokens T of a length-L sequence under this map: L*K for a dense map, the kept positions
 * for a sampled one (which accepts only its own L).  -1 on a bad argument. */
int64_t peagle_tilemap_tokens(const peagle_tilemap_t* tm, int32_t L);

/*
 * Rotary position embedding around the attention step.  The drafter follows the LLaMA 3
 * architecture with RoPE (Sec. 2), and depth d predicts the token d+1 ahead of its anchor (Sec. 3),
 * so the stored token (anchor i, depth d) stands at sequence position p = i + d; positions restart
 * with every sequence of a packed batch.  Feature pair (j, j + D/2) of every head vector of Q and K
 * turns by the angle p * base^(-2j/D) (half-split pairing; LLaMA 3 uses base = 500000).
 *
 * peagle_rope_positions: number of positions a table must cover for a length-L problem under this
 * map (largest position + 1: L + K - 1 for a dense map); -1 on a bad argument.
 *
 * peagle_rope_table: fills table (device, fp32 [n_pos][2][D/2]: per position D/2 cosines, then D/2
 * sines) on `stream`; angles are formed and reduced in double precision.  Built once per
 * (base, D, n_pos) and reused, like the tile map.  EINVAL unless base > 1 and n_pos >= 1.
 */
int32_t peagle_rope_positions(const peagle_tilemap_t* tm, int32_t L);
/* Position id of every stored token of a length-L problem: pos_out (host, int32[T]). */
int peagle_rope_position_ids(const peagle_tilemap_t* tm, int32_t L, int32_t* pos_out);
int peagle_rope_table(float base, int32_t D, int32_t n_pos, float* table, void* stream);

/*
 * out = R x (inverse = 0) or R^T x (inverse = 1) for a tensor of the map's tokens:
 *   x, out      device, bf16 [T, H, D] (H heads; out may not overlap x unless equal to it)
 *   rope_table  device, from peagle_rope_table with n_pos >= peagle_rope_positions (else ESHAPE)
 * fp32 arithmetic, one rounding to bf16.  Exposed for tests and for callers that keep rotated copies.
 */
int peagle_rope_rotate(const peagle_tilemap_t* tm, const peagle_shape_t* shape, const void* x, int32_t H,
                       const float* rope_table, int32_t n_pos, int32_t inverse, void* out, void* stream);

/* Bytes of device scratch peagle_attn_step_partitioned_rope needs: the attention workspace plus
 * rotated bf16 copies of Q and K. */
size_t peagle_rope_workspace_bytes(const peagle_tilemap_t* tm, const peagle_shape_t* shape);

/*
 * peagle_attn_step_partitioned on unrotated Q and K: both are rotated by their tokens' positions
 * (one streaming pass each, into the workspace), every segment's forward and backward run on the
 * rotated copies, and dQ, dK are returned with respect to the unrotated inputs: the gradient
 * vectors are turned back (R^T) in fp32 inside the kernels that store them (dQ kernel, chain-key
 * epilogue of the dK/dV kernel, summation of the depth-0 partials), so dk_acc stays in the
 * unrotated frame across segments and calls.  Every other argument, and the dK/dV accumulation
 * rule, are those of peagle_attn_step_partitioned; workspace >= peagle_rope_workspace_bytes().
 */
int peagle_attn_step_partitioned_rope(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg_begin,
                                      int32_t seg_end, const void* q, const void* k, const void* v,
                                      const void* d_o, const float* rope_table, int32_t n_pos, void* o, float* lse,
                                      void* dq, float* dk_acc, float* dv_acc, void* dk_bf16, void* dv_bf16,
                                      void* workspace, size_t ws_bytes, void* stream);

/*
 * The rotary step as the first drafter layer sees it.  Every multi-token position is fed the same
 * input - the shared hidden state and the mask-token embedding (Sec. 2) - so before the rotation the
 * keys of all positions of depth >= 1 are one vector per KV head, and their values one vector; only
 * the depth-0 positions, the first L stored tokens of any map, have keys and values of their own.
 * The caller passes those and the two shared vectors instead of [T, Hkv, D] tensors, and gets the
 * gradients in the same form.  All S segments run (in order, dK/dV accumulated across them).
 *
 *   q, d_o, o, dq   device, bf16 [T, Hq, D] as in peagle_attn_step_partitioned_rope; lse fp32 [Hq, T]
 *   k0, v0          device, bf16 [L, Hkv, D]: unrotated keys / values of the depth-0 positions
 *   k_shared, v_shared   device, bf16 [Hkv, D]: the unrotated key / value of every other position
 *   dk0, dv0        device, fp32 [L, Hkv, D] (out)
 *   dk_shared, dv_shared   device, fp32 [Hkv, D] (out): sums over all positions of depth >= 1 (for the
 *                   keys, of the gradients turned back to the unrotated frame); deterministic
 *   workspace       device, >= peagle_rope_shared_workspace_bytes(): besides the rotary workspace it holds
 *                   one row of Hkv x D partial sums of dK and of dV per wave of the workgroups that own the
 *                   chain keys (a few MB)
 * The keys are expanded and rotated in one pass (each chain row reads the shared vector, not HBM rows
 * of its own).  The values are not expanded at D = 64: the kernels read every chain key's value row
 * from v_shared (at D = 128 the forward and dQ kernels have no registers for that and get an expanded V
 * in the workspace).  No [T, Hkv, D] gradient tensor exists either: the depth-0 keys' dK / dV are written to
 * dk0 / dv0 directly, and the chain keys' dK (turned back to the unrotated frame key by key) and dV are
 * summed over each wave's 32 keys inside the dK/dV kernel, then over the waves by a two-stage
 * reduction in a fixed order.
 */
size_t peagle_rope_shared_workspace_bytes(const peagle_tilemap_t* tm, const peagle_shape_t* shape);
int peagle_attn_step_rope_shared(const peagle_tilemap_t* tm, const peagle_shape_t* shape, const void* q,
                                 const void* k0, const void* k_shared, const void* v0, const void* v_shared,
                                 const void* d_o, const float* rope_table, int32_t n_pos, void* o, float* lse,
                                 void* dq, float* dk0, float* dv0, float* dk_shared, float* dv_shared,
                                 void* workspace, size_t ws_bytes, void* stream);

/*
 * Inference-side parallel drafting (Sec. 2: the drafter produces all K draft tokens in a single
 * forward pass; the serving experiments run K = 3, 5, 7 at concurrency 2-4).  One drafting step adds K
 * positions after a request's cached context of n tokens: the next-token position (depth 0) and K-1
 * multi-token positions (depths 1..K-1), all of the anchor that follows the context.  They are the
 * last anchor's rows of the parallel-prediction mask (Sec. 3): the row of depth d sees the n cached
 * keys and the new keys of depth 0..d.  This call computes that attention for C requests at once.
 *
 * The cache is paged: page = PEAGLE_PAGE_TOKENS (64) consecutive tokens of one request, all KV heads.
 *
 *   shape        C requests (<= 65535), K new positions each (<= 64), Hq / Hkv heads (Hq % Hkv == 0,
 *                K * Hq/Hkv <= 128), D in {64, 128}, scale > 0, n_pages pages in the pools, max_pages
 *                block-table columns (<= 2^24); anything else: EINVAL / EUNSUPPORTED before any launch
 *   q_new        device, bf16 [C, K, Hq, D]          k_new, v_new  device, bf16 [C, K, Hkv, D]
 *   k_pages, v_pages   device, bf16 [n_pages, Hkv, 64, D]  (the tail of a request's last page may hold
 *                anything: it is never used in arithmetic)
 *   block_table  device, int32 [C, max_pages]: page holding tokens [64 b, 64 b + 64) of request c
 *   ctx_len      device, int32 [C]: cached tokens n of each request, 0 <= n <= 64 * max_pages
 *   o            device, bf16 [C, K, Hq, D] (out)    lse  device, fp32 [C, Hq, K] (out; natural log)
 *   status       device, int32 [C] or NULL (out): 1 if a block-table entry the request uses is outside
 *                [0, n_pages) or its ctx_len is out of range (such blocks are skipped, the length is
 *                clamped, nothing is read out of bounds), else 0
 *   workspace    device, >= peagle_draft_decode_workspace_bytes(); contents undefined before and after
 *
 * The context of every request is cut into peagle_draft_decode_splits() pieces that run in
 * parallel (one workgroup per piece, KV head and request) and are merged by a second launch.
 * Nothing is allocated and nothing is copied to the host: the call can sit in a serving loop.
 */
#define PEAGLE_PAGE_TOKENS 64
typedef struct peagle_decode_shape {
  int32_t C, K, Hq, Hkv, D;
  float scale;
  int32_t n_pages, max_pages;
} peagle_decode_shape_t;
int32_t peagle_draft_decode_splits(const peagle_decode_shape_t* shape);
size_t peagle_draft_decode_workspace_bytes(const peagle_decode_shape_t* shape);
int peagle_draft_decode(const peagle_decode_shape_t* shape, const void* q_new, const void* k_new, const void* v_new,
                        const void* k_pages, const void* v_pages, const int32_t* block_table, const int32_t* ctx_len,
                        void* o, float* lse, int32_t* status, void* workspace, size_t ws_bytes, void* stream);

/*
 * The same drafting step for callers that cannot allocate or hand over device memory for scratch:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The partial
 * records live in an array inside the loaded library (PEAGLE_STATIC_SCRATCH_BYTES per GPU, held until
 * the process ends) instead of a caller workspace; every other argument is as in peagle_draft_decode
 * and the results are bit-identical to it.  Shapes whose records need more than that
 * (peagle_draft_decode_workspace_bytes() > PEAGLE_STATIC_SCRATCH_BYTES) are rejected with
 * PEAGLE_EWORKSPACE before any launch.  The call allocates and frees nothing.  All calls on one GPU
 * share that GPU's array: calls that overlap there (two streams, two threads) race; calls on one
 * stream are ordered and safe.  The array keeps the previous call's records; the kernels overwrite
 * every record they later read, so nothing needs clearing.
 */
#define PEAGLE_STATIC_SCRATCH_BYTES (32u << 20)
int peagle_draft_decode_static(const peagle_decode_shape_t* shape, const void* q_new, const void* k_new,
                               const void* v_new, const void* k_pages, const void* v_pages,
                               const int32_t* block_table, const int32_t* ctx_len, void* o, float* lse,
                               int32_t* status, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* peagle_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PEAGLE_H */
