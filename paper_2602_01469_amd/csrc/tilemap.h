// Internal representation of the tile map (host side) and the device view handed to kernels.
//
// Geometry (see include/peagle.h): a row tile is A = 128/K anchors at all K depths (dense map) or a
// run of anchors whose kept positions fill 128 rows (sampled / packed maps); key tiles are 64 wide
// and come from two streams (depth-0 anchors, and the chain positions of a row tile's own
// anchors).  The classification follows the parallel-prediction mask of Sec. 3 of the paper.
#pragma once

#include <cstdint>
#include <vector>

#include "peagle.h"

namespace peagle {

constexpr int kRowsPerTile = 128;
constexpr int kKeysPerTile = 64;
constexpr int kMaskWordsPerRow = kKeysPerTile / 32;                   // 2 x u32 per row
constexpr int kMaskWords = kRowsPerTile * kMaskWordsPerRow;           // 256 x u32 = 1 KiB per mask

struct TileEntry {
  int32_t tile;     // key-tile id in the row-tile lists, row-tile id in the key-tile lists
  int32_t mask_id;  // -1: every element of the pair is visible; >= 0: index into the mask pool.  Key-tile lists
                    // of packed maps also use INT32_MIN (listed for the pair's other tile only: nothing to do)
                    // and -2 - a (visible for keys with anchor >= a: the row tile's sequence starts at a)
};

// Pointers into device memory; passed to kernels by value.
struct DeviceTileMap {
  const int32_t* row_ptr;     // [n_row_tiles + 1]  offsets into row_entries
  const TileEntry* row_entries;
  const int32_t* row_lead;    // [n_row_tiles]  length of the leading run of full entries in each row tile's list
  const int32_t* key_ptr;     // [n_key_tiles + 1]  offsets into key_entries (row tiles ascending)
  const TileEntry* key_entries;
  const int32_t* key_seg_ptr; // [n_key_tiles][S + 1]  offsets into key_entries: where each segment's row tiles start
  const uint32_t* masks;      // [n_masks][128][2]: bit k%32 of word k/32 of row r: row r sees key k
  const uint32_t* masks_by_key;  // [n_masks][64][4]: the same bits key-major (bit r%32 of word r/32 of key k)
  const void* zeros;          // 256 zero bytes: source of rows that do not exist, for direct-to-LDS loads
  const int32_t* row_tok;     // sampled maps only (else null): [n_row_tiles][128] token of each row, -1 = no row
  const int32_t* chain_tok;   // sampled maps only: [n_row_tiles * n_csub][64] token of each chain key, -1 = none
  const int32_t* tok_posid;   // sampled maps only: [T] sequence position (anchor - sequence start + depth) of each token
  int32_t A, K, S, n_row_tiles, n_d0, n_csub, n_key_tiles;
};

}  // namespace peagle

struct peagle_tilemap {
  int32_t L_max = 0, K = 0, S = 0, A = 0;       // A = 0 for a sampled map (anchors per row tile vary)
  int32_t sampled = 0;                           // built from a drop-token sampled position set
  int64_t T_tokens = 0;                          // stored tokens of a length-L_max sequence
  std::vector<int32_t> seg_rt;                   // [S+1] first row tile of each segment
  std::vector<int32_t> seg_key_lo;               // [S] first depth-0 key (anchor) a segment's rows can see (packed batches)
  std::vector<int32_t> row_tok, chain_tok;       // explicit token lists of a sampled map (empty for a dense one)
  std::vector<int32_t> key_side_id;              // per row entry, packed maps only: the id the key tile -> row tile
                                                 // list carries when it differs from the row side (see finish_map)
  std::vector<int64_t> tok_pos;                  // sampled map, host only: token -> row tile * 128 + row
  std::vector<int32_t> tok_posid;                // sampled map: token -> sequence position (rotary embedding)
  int32_t max_posid = 0;                         // largest entry of tok_posid
  int32_t n_row_tiles = 0, n_d0 = 0, n_csub = 0, n_key_tiles = 0;
  std::vector<int32_t> seg_bounds;               // [S+1] anchors
  std::vector<int32_t> row_ptr;
  std::vector<int32_t> row_lead;                 // leading full entries per row tile
  std::vector<peagle::TileEntry> row_entries;
  std::vector<int32_t> key_ptr;
  std::vector<peagle::TileEntry> key_entries;
  std::vector<int32_t> key_seg_ptr;              // n_key_tiles * (S+1)
  std::vector<uint32_t> masks;                   // n_masks * kMaskWords
  int64_t n_full = 0, n_partial = 0;
  int32_t n_masks = 0;
  int32_t device = -1;
  void* dev_blob = nullptr;                      // one allocation holding all device arrays
  void* staging = nullptr;                       // pinned host image of the blob (source of the upload copy)
  void* copy_done = nullptr;                     // hipEvent_t recorded after the last upload copy
  int64_t dev_capacity = 0;                      // bytes allocated for dev_blob and staging
  int64_t dev_bytes = 0;                         // bytes in use
  peagle::DeviceTileMap dview{};
};

namespace peagle {

// Anchor range [lo, hi) of a segment clipped to a length-L problem, and the row tiles covering it.
struct SegRange {
  int32_t a_lo, a_hi, rt_lo, rt_hi;
  int32_t key_lo;      // first depth-0 key any of the rows can see (0 unless the map packs several sequences)
  int32_t s_lo, s_hi;  // segment boundary indices spanned: [bounds[s_lo], bounds[s_hi])
  int32_t cropped;     // the range ends before bounds[s_hi] (L < L_max cuts it short)
};
int resolve_segment(const peagle_tilemap* tm, int32_t L, int32_t seg, SegRange* out);

}  // namespace peagle
