// Mask -> tile map (amortized mask construction, Sec. 3.1 of the paper; segment boundaries of
// Sec. 3.2).  Host code only, apart from the one upload of the finished map.
//
// The builder never touches the O((nK)^2) element mask: every (row tile, key tile) pair is
// classified with interval tests, and only the O(1) distinct partial patterns are expanded
// element by element (from the visibility rule) into the de-duplicated mask pool.
#include "tilemap.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <unordered_map>

using peagle::kKeysPerTile;
using peagle::kMaskWords;
using peagle::kMaskWordsPerRow;
using peagle::kRowsPerTile;
using peagle::TileEntry;

namespace {

// Visibility rule of the parallel-prediction mask in anchor coordinates (Sec. 3; Sec. 3.2,
// dependency of (p, d) on (p-1, d-1)): depth-0 keys are causal in the anchor, keys of depth
// e >= 1 are visible only on the row's own anchor and only up to the row's depth.
inline bool sees(int64_t i, int d, int64_t j, int e) {
  return e == 0 ? (j <= i) : (j == i && e <= d);
}

struct MaskPool {
  std::map<std::vector<uint32_t>, int32_t> index;
  std::vector<uint32_t>* storage;
  int32_t intern(const std::vector<uint32_t>& bits) {
    auto it = index.find(bits);
    if (it != index.end()) return it->second;
    int32_t id = (int32_t)index.size();
    index.emplace(bits, id);
    storage->insert(storage->end(), bits.begin(), bits.end());
    return id;
  }
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

namespace {

// Second half of both builders, host part: key tile -> row tile lists and per-segment offsets.
void build_key_lists(peagle_tilemap* tm) {
  // key tile -> row tiles (ascending), same mask ids
  std::vector<std::vector<TileEntry>> lists(tm->n_key_tiles);
  for (int32_t R = 0; R < tm->n_row_tiles; ++R)
    for (int32_t e = tm->row_ptr[R]; e < tm->row_ptr[R + 1]; ++e) {
      const TileEntry& en = tm->row_entries[e];
      // Key side of a pair that is partial only because the row tile's sequence starts inside the key
      // tile: the keys of the earlier sequence are separate lanes of the dK/dV kernel, which drops
      // them by anchor (id -2 - first anchor of the sequence) instead of reading a bitmask.
      const int32_t id = tm->key_side_id.empty() ? en.mask_id : tm->key_side_id[e];
      lists[en.tile].push_back(TileEntry{R, id});
    }
  // The dK/dV kernel walks depth-0 key tiles in pairs (2m, 2m+1) along the list of the first and
  // expects the list of the second to be a suffix of it.  That holds for one sequence (a row tile
  // that sees tile 2m+1 has anchors past it and sees 2m as well).  In a packed batch a later
  // sequence may start inside or after tile 2m: its row tiles see 2m+1 only, and they come after
  // every row tile that sees 2m - they are appended to the list of 2m with the id INT32_MIN, which
  // tells the waves that own the keys of 2m to sit the iteration out.
  for (int32_t t0 = 0; t0 + 1 < tm->n_d0; t0 += 2) {
    std::vector<TileEntry>& first = lists[t0];
    const std::vector<TileEntry>& second = lists[t0 + 1];
    const int32_t last_first = first.empty() ? -1 : first.back().tile;
    for (const TileEntry& en : second)
      if (en.tile > last_first) first.push_back(TileEntry{en.tile, INT32_MIN});
  }
  tm->key_ptr.assign(tm->n_key_tiles + 1, 0);
  for (int32_t t = 0; t < tm->n_key_tiles; ++t) tm->key_ptr[t + 1] = tm->key_ptr[t] + (int32_t)lists[t].size();
  tm->key_entries.clear();
  tm->key_entries.reserve(tm->key_ptr[tm->n_key_tiles]);
  for (int32_t t = 0; t < tm->n_key_tiles; ++t) tm->key_entries.insert(tm->key_entries.end(), lists[t].begin(), lists[t].end());

  // per key tile: where the row tiles of each segment start inside its list
  tm->key_seg_ptr.resize((size_t)tm->n_key_tiles * (tm->S + 1));
  for (int32_t t = 0; t < tm->n_key_tiles; ++t) {
    int32_t e = tm->key_ptr[t];
    for (int32_t sg = 0; sg <= tm->S; ++sg) {
      const int32_t first_rt = tm->seg_rt[sg];
      while (e < tm->key_ptr[t + 1] && tm->key_entries[e].tile < first_rt) ++e;
      tm->key_seg_ptr[(size_t)t * (tm->S + 1) + sg] = e;
    }
  }

}

// Device copy of a finished map: all arrays packed into one blob, staged in pinned host memory and
// sent with a single copy on `stream`.  The device allocation and the staging buffer are kept in
// the handle and reused while they are large enough, so that rebuilding a map (a new sample every
// training step) allocates nothing.  With wait = true the copy has completed on return.
int upload_map(peagle_tilemap* tm, hipStream_t stream, bool wait) {
  if (tm->device < 0) return PEAGLE_OK;
  int prev = -1;
  if (hipGetDevice(&prev) != hipSuccess || hipSetDevice(tm->device) != hipSuccess) return PEAGLE_EHIP;
  constexpr int kArrays = 12;
  static const char kZeros[256] = {0};
  const size_t sz[kArrays] = {tm->row_ptr.size() * sizeof(int32_t), tm->row_entries.size() * sizeof(TileEntry),
                              tm->key_ptr.size() * sizeof(int32_t), tm->key_entries.size() * sizeof(TileEntry),
                              tm->masks.size() * sizeof(uint32_t), tm->key_seg_ptr.size() * sizeof(int32_t),
                              sizeof(kZeros), tm->row_lead.size() * sizeof(int32_t),
                              tm->row_tok.size() * sizeof(int32_t), tm->chain_tok.size() * sizeof(int32_t),
                              tm->tok_posid.size() * sizeof(int32_t), tm->masks.size() * sizeof(uint32_t)};
  const void* src[kArrays] = {tm->row_ptr.data(), tm->row_entries.data(), tm->key_ptr.data(),
                              tm->key_entries.data(), tm->masks.data(), tm->key_seg_ptr.data(), kZeros,
                              tm->row_lead.data(), tm->row_tok.data(), tm->chain_tok.data(), tm->tok_posid.data(),
                              nullptr /* the key-major masks are written into the staging image below */};
  size_t off[kArrays], total = 0;
  for (int i = 0; i < kArrays; ++i) {
    off[i] = total;
    total += align256(sz[i] ? sz[i] : 4);
  }
  hipError_t err = hipSuccess;
  if (tm->copy_done) err = hipEventSynchronize((hipEvent_t)tm->copy_done);  // the staging buffer is free again
  if (err == hipSuccess && total > (size_t)tm->dev_capacity) {
    // grow with headroom; the old blob may still be read by kernels already enqueued: wait for them
    const size_t cap = total + total / 4;
    if (tm->dev_blob) {
      err = hipDeviceSynchronize();
      (void)hipFree(tm->dev_blob);
      (void)hipHostFree(tm->staging);
      tm->dev_blob = tm->staging = nullptr;
      tm->dev_capacity = 0;
    }
    if (err == hipSuccess) err = hipMalloc(&tm->dev_blob, cap);
    if (err == hipSuccess) err = hipHostMalloc(&tm->staging, cap, hipHostMallocDefault);
    if (err == hipSuccess) tm->dev_capacity = (int64_t)cap;
  }
  if (err == hipSuccess && !tm->copy_done) {
    hipEvent_t ev = nullptr;
    err = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    tm->copy_done = ev;
  }
  if (err == hipSuccess) {
    for (int i = 0; i < kArrays; ++i)
      if (sz[i] && src[i]) std::memcpy((char*)tm->staging + off[i], src[i], sz[i]);
    // key-major copy of every mask for the dK/dV kernel, whose lanes own keys: word r/32 of key k has bit r%32
    // set iff row r sees key k
    uint32_t* mt = (uint32_t*)((char*)tm->staging + off[11]);
    for (int32_t m = 0; m < tm->n_masks; ++m)
      for (int k = 0; k < kKeysPerTile; ++k)
        for (int w = 0; w < kRowsPerTile / 32; ++w) {
          uint32_t bits = 0;
          for (int b = 0; b < 32; ++b) {
            const uint32_t rw = tm->masks[(size_t)m * kMaskWords + (size_t)(w * 32 + b) * kMaskWordsPerRow + k / 32];
            bits |= ((rw >> (k % 32)) & 1u) << b;
          }
          mt[(size_t)m * kMaskWords + (size_t)k * (kRowsPerTile / 32) + w] = bits;
        }
    err = hipMemcpyAsync(tm->dev_blob, tm->staging, total, hipMemcpyHostToDevice, stream);
  }
  if (err == hipSuccess) err = hipEventRecord((hipEvent_t)tm->copy_done, stream);
  if (err == hipSuccess && wait) err = hipEventSynchronize((hipEvent_t)tm->copy_done);
  (void)hipSetDevice(prev);
  if (err != hipSuccess) return PEAGLE_EHIP;
  tm->dev_bytes = (int64_t)total;
  char* base = (char*)tm->dev_blob;
  tm->dview.row_ptr = (const int32_t*)(base + off[0]);
  tm->dview.row_entries = (const TileEntry*)(base + off[1]);
  tm->dview.key_ptr = (const int32_t*)(base + off[2]);
  tm->dview.key_entries = (const TileEntry*)(base + off[3]);
  tm->dview.masks = (const uint32_t*)(base + off[4]);
  tm->dview.key_seg_ptr = (const int32_t*)(base + off[5]);
  tm->dview.zeros = base + off[6];
  tm->dview.row_lead = (const int32_t*)(base + off[7]);
  tm->dview.row_tok = tm->row_tok.empty() ? nullptr : (const int32_t*)(base + off[8]);
  tm->dview.chain_tok = tm->chain_tok.empty() ? nullptr : (const int32_t*)(base + off[9]);
  tm->dview.tok_posid = tm->tok_posid.empty() ? nullptr : (const int32_t*)(base + off[10]);
  tm->dview.masks_by_key = (const uint32_t*)(base + off[11]);
  tm->dview.A = tm->A;
  tm->dview.K = tm->K;
  tm->dview.S = tm->S;
  tm->dview.n_row_tiles = tm->n_row_tiles;
  tm->dview.n_d0 = tm->n_d0;
  tm->dview.n_csub = tm->n_csub;
  tm->dview.n_key_tiles = tm->n_key_tiles;
  return PEAGLE_OK;
}

void release_device(peagle_tilemap* tm) {
  if (tm->device < 0 || (!tm->dev_blob && !tm->staging && !tm->copy_done)) return;
  int prev = -1;
  if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(tm->device) == hipSuccess) {
    if (tm->copy_done) {
      (void)hipEventSynchronize((hipEvent_t)tm->copy_done);
      (void)hipEventDestroy((hipEvent_t)tm->copy_done);
    }
    if (tm->dev_blob) (void)hipFree(tm->dev_blob);
    if (tm->staging) (void)hipHostFree(tm->staging);
    (void)hipSetDevice(prev);
  }
  tm->dev_blob = tm->staging = nullptr;
  tm->copy_done = nullptr;
  tm->dev_capacity = 0;
}

// Common tail of the builders.  Takes ownership of tm (released on failure).
int finish_map(peagle_tilemap* tm, int32_t device, peagle_tilemap_t** out) {
  build_key_lists(tm);
  tm->device = device;
  const int rc = upload_map(tm, nullptr, true);
  if (rc != PEAGLE_OK) {
    release_device(tm);
    delete tm;
    return rc;
  }
  *out = tm;
  return PEAGLE_OK;
}

}  // namespace

extern "C" int peagle_build_tilemap(int32_t L_max, int32_t K, const int32_t* seg_bounds, int32_t S, int32_t device,
                                    peagle_tilemap_t** out) {
  if (!out) return PEAGLE_ENULL;
  *out = nullptr;
  if (L_max < 1 || S < 1 || K < 1) return PEAGLE_EINVAL;
  if (K > kRowsPerTile) return PEAGLE_EUNSUPPORTED;
  if ((int64_t)L_max * K > (int64_t)1 << 30) return PEAGLE_EUNSUPPORTED;
  if (!seg_bounds && S != 1) return PEAGLE_ENULL;
  const int32_t A = kRowsPerTile / K;

  peagle_tilemap* tm = new (std::nothrow) peagle_tilemap();
  if (!tm) return PEAGLE_EINVAL;
  tm->L_max = L_max;
  tm->K = K;
  tm->S = S;
  tm->A = A;
  if (seg_bounds) {
    tm->seg_bounds.assign(seg_bounds, seg_bounds + S + 1);
  } else {
    tm->seg_bounds = {0, L_max};
  }
  const std::vector<int32_t>& b = tm->seg_bounds;
  bool ok = b[0] == 0 && b[S] == L_max;
  for (int s = 0; s < S && ok; ++s) ok = b[s] < b[s + 1];
  for (int s = 1; s < S && ok; ++s) ok = (b[s] % A) == 0;
  if (!ok) {
    delete tm;
    return PEAGLE_EBOUNDS;
  }

  tm->n_row_tiles = (L_max + A - 1) / A;
  tm->n_d0 = (L_max + kKeysPerTile - 1) / kKeysPerTile;
  const int32_t chain_keys = A * (K - 1);
  tm->n_csub = (chain_keys + kKeysPerTile - 1) / kKeysPerTile;
  const int64_t n_kt = (int64_t)tm->n_d0 + (int64_t)tm->n_row_tiles * tm->n_csub;
  if (n_kt > (int64_t)1 << 30) {
    delete tm;
    return PEAGLE_EUNSUPPORTED;
  }
  tm->n_key_tiles = (int32_t)n_kt;

  MaskPool pool;
  pool.storage = &tm->masks;
  std::vector<uint32_t> bits(kMaskWords);
  const int rows_used = A * K;

  tm->row_ptr.assign(tm->n_row_tiles + 1, 0);
  for (int32_t R = 0; R < tm->n_row_tiles; ++R) {
    const int64_t i0 = (int64_t)R * A;        // first anchor of the row tile
    const int64_t i1 = i0 + A - 1;            // last anchor (position-invariant: not clipped to L_max)
    // depth-0 stream: key tile c holds anchors [64c, 64c+63]
    for (int32_t c = 0; c < tm->n_d0; ++c) {
      const int64_t j0 = (int64_t)c * kKeysPerTile, j1 = j0 + kKeysPerTile - 1;
      if (j0 > i1) break;                     // every key is in the future of every row: empty
      TileEntry en{c, -1};
      if (j1 <= i0) {                         // every key is visible to every row: full
        ++tm->n_full;
      } else {
        std::fill(bits.begin(), bits.end(), 0u);
        for (int r = 0; r < rows_used; ++r) {
          const int d = r / A;
          const int64_t i = i0 + r % A;
          for (int kk = 0; kk < kKeysPerTile; ++kk)
            if (sees(i, d, j0 + kk, 0)) bits[r * kMaskWordsPerRow + kk / 32] |= 1u << (kk % 32);
        }
        en.mask_id = pool.intern(bits);
        ++tm->n_partial;
      }
      tm->row_entries.push_back(en);
    }
    // chain stream: key kk of the stream is depth 1 + kk/A, anchor i0 + kk%A
    for (int32_t s = 0; s < tm->n_csub; ++s) {
      std::fill(bits.begin(), bits.end(), 0u);
      bool any = false;
      for (int r = 0; r < rows_used; ++r) {
        const int d = r / A;
        const int64_t i = i0 + r % A;
        for (int kk = 0; kk < kKeysPerTile; ++kk) {
          const int ck = s * kKeysPerTile + kk;
          if (ck >= chain_keys) break;
          if (sees(i, d, i0 + ck % A, 1 + ck / A)) {
            bits[r * kMaskWordsPerRow + kk / 32] |= 1u << (kk % 32);
            any = true;
          }
        }
      }
      if (!any) continue;
      const int32_t kt = tm->n_d0 + R * tm->n_csub + s;
      tm->row_entries.push_back(TileEntry{kt, pool.intern(bits)});
      ++tm->n_partial;
    }
    tm->row_ptr[R + 1] = (int32_t)tm->row_entries.size();
    int32_t lead = 0;
    for (int32_t e = tm->row_ptr[R]; e < tm->row_ptr[R + 1] && tm->row_entries[e].mask_id < 0; ++e) ++lead;
    tm->row_lead.push_back(lead);
  }
  tm->n_masks = (int32_t)pool.index.size();
  tm->seg_rt.resize(S + 1);
  for (int32_t sg = 0; sg <= S; ++sg) tm->seg_rt[sg] = sg == S ? tm->n_row_tiles : b[sg] / A;
  tm->T_tokens = (int64_t)L_max * K;
  return finish_map(tm, device, out);
}

extern "C" void peagle_tilemap_destroy(peagle_tilemap_t* tm) {
  if (!tm) return;
  release_device(tm);
  delete tm;
}

// Tile map of a drop-token sampled sequence (Conditional Drop-token sampling, PARD paragraph of
// Sec. 3; kept positions are nested per anchor, Sec. 3.2 Challenge 2).  Same structure as the
// dense map, with three differences: a row tile is a run of consecutive anchors packed greedily
// until its kept positions would exceed 128 rows (never across a segment boundary), so every
// tile is full of rows that exist; rows and chain keys are named by explicit token lists; the
// partial masks depend on the sample and are built per tile from the same visibility rule.
extern "C" int peagle_build_tilemap_sampled(const int32_t* depth_count, int32_t L, int32_t K,
                                            const int32_t* seg_bounds, int32_t S, int32_t assignment,
                                            int32_t device, peagle_tilemap_t** out) {
  if (out) *out = nullptr;
  if (!depth_count) return PEAGLE_ENULL;
  return peagle_build_tilemap_packed(depth_count, L, K, nullptr, 1, seg_bounds, S, assignment, device, out);
}

namespace {

// Fills the host arrays of `tm` (any previous content is dropped) for the given position set; the
// device side is untouched.  Every argument is checked before tm is modified.
int fill_packed(peagle_tilemap* tm, const int32_t* depth_count_in, int32_t L, int32_t K, const int32_t* seq_start_in,
                int32_t n_seq, const int32_t* seg_bounds, int32_t S, int32_t assignment) {
  if (L < 1 || S < 1 || K < 1 || n_seq < 1) return PEAGLE_EINVAL;
  if (assignment != PEAGLE_ASSIGN_BY_ANCHOR && assignment != PEAGLE_ASSIGN_ALGORITHM1) return PEAGLE_EINVAL;
  if (K > kRowsPerTile) return PEAGLE_EUNSUPPORTED;
  if ((int64_t)L * K > (int64_t)1 << 30) return PEAGLE_EUNSUPPORTED;
  if (!seg_bounds && S != 1) return PEAGLE_ENULL;
  if (!seq_start_in && n_seq != 1) return PEAGLE_ENULL;
  std::vector<int32_t> all_depths;
  if (!depth_count_in) all_depths.assign(L, K);
  const int32_t* depth_count = depth_count_in ? depth_count_in : all_depths.data();
  for (int32_t i = 0; i < L; ++i)
    if (depth_count[i] < 1 || depth_count[i] > K) return PEAGLE_EINVAL;
  std::vector<int32_t> seq_start(n_seq + 1);
  if (seq_start_in) seq_start.assign(seq_start_in, seq_start_in + n_seq + 1);
  else seq_start = {0, L};
  {
    bool ok = seq_start[0] == 0 && seq_start[n_seq] == L;
    for (int q = 0; q < n_seq && ok; ++q) ok = seq_start[q] < seq_start[q + 1];
    if (!ok) return PEAGLE_EBOUNDS;
  }
  std::vector<int32_t> b;
  if (seg_bounds) b.assign(seg_bounds, seg_bounds + S + 1);
  else b = {0, L};
  {
    bool ok = b[0] == 0 && b[S] == L;
    for (int s = 0; s < S && ok; ++s) ok = b[s] < b[s + 1];
    if (!ok) return PEAGLE_EBOUNDS;
  }
  // first and one-past-last anchor of the sequence every anchor belongs to
  std::vector<int32_t> seq_lo(L), seq_hi(L);
  for (int32_t q = 0; q < n_seq; ++q)
    for (int32_t i = seq_start[q]; i < seq_start[q + 1]; ++i) {
      seq_lo[i] = seq_start[q];
      seq_hi[i] = seq_start[q + 1];
    }

  tm->L_max = L;
  tm->K = K;
  tm->S = S;
  tm->A = 0;  // anchors per row tile vary
  tm->sampled = 1;
  tm->seg_bounds = b;
  tm->n_full = tm->n_partial = 0;
  tm->n_masks = 0;
  tm->row_entries.clear();
  tm->row_lead.clear();
  tm->masks.clear();
  tm->key_side_id.clear();

  // token of (depth, anchor): depth-major storage, kept anchors ascending; its sequence position is
  // the anchor's offset in its sequence plus the depth (depth g predicts the token g+1 ahead, Sec. 3)
  std::vector<int32_t> tok_of((size_t)L * K, -1);
  int32_t next = 0;
  tm->tok_posid.clear();
  tm->max_posid = 0;
  for (int32_t g = 0; g < K; ++g)
    for (int32_t i = 0; i < L; ++i)
      if (depth_count[i] > g) {
        tok_of[(size_t)g * L + i] = next++;
        tm->tok_posid.push_back(i - seq_lo[i] + g);
        tm->max_posid = std::max(tm->max_posid, i - seq_lo[i] + g);
      }
  tm->T_tokens = next;
  tm->tok_pos.assign(next, -1);

  // Segment of an anchor's rows.  Depth 0 always goes by the anchor.  The deeper rows of anchor i
  // either follow it (by anchor), or go where Algorithm 1 puts them: the depth-1 position is
  // p = i + 1 and is assigned by its own position, deeper depths inherit from (p-1, g-1), so the
  // whole chain of anchor i lands in the segment that holds position i + 1 (the anchor's own
  // segment if i + 1 is past its sequence).
  std::vector<int32_t> seg_of_pos(L + 1);
  for (int32_t sg = 0; sg < S; ++sg)
    for (int32_t i = b[sg]; i < b[sg + 1]; ++i) seg_of_pos[i] = sg;
  seg_of_pos[L] = S - 1;
  auto chain_seg = [&](int32_t i) {  // position i + 1 past the anchor's own sequence: its last segment
    return assignment == PEAGLE_ASSIGN_ALGORITHM1 && i + 1 < seq_hi[i] ? seg_of_pos[i + 1] : seg_of_pos[i];
  };
  auto rows_in = [&](int32_t i, int32_t sg) {  // rows of anchor i computed in segment sg
    return (seg_of_pos[i] == sg ? 1 : 0) + (chain_seg(i) == sg ? depth_count[i] - 1 : 0);
  };

  // greedy packing of anchors into row tiles, one segment at a time
  std::vector<int32_t> tile_a0, tile_a1, tile_seg;  // anchors [a0, a1) of each row tile and its segment
  tm->seg_rt.assign(S + 1, 0);
  for (int32_t sg = 0; sg < S; ++sg) {
    tm->seg_rt[sg] = (int32_t)tile_a0.size();
    int32_t a = b[sg] > 0 ? b[sg] - 1 : 0;  // the previous anchor's chain may belong here
    while (a < b[sg + 1]) {
      if (rows_in(a, sg) == 0) {
        ++a;
        continue;
      }
      int32_t rows = 0, e = a;
      while (e < b[sg + 1] && e < seq_hi[a] && rows + rows_in(e, sg) <= kRowsPerTile) rows += rows_in(e++, sg);
      while (e > a && rows_in(e - 1, sg) == 0) --e;  // no trailing anchors without rows
      tile_a0.push_back(a);
      tile_a1.push_back(e);
      tile_seg.push_back(sg);
      a = e;
    }
  }
  tm->n_row_tiles = (int32_t)tile_a0.size();
  tm->seg_rt[S] = tm->n_row_tiles;
  // first depth-0 key a segment's rows can see: the start of the sequence of its first row's anchor
  tm->seg_key_lo.assign(S, 0);
  for (int32_t sg = 0; sg < S; ++sg) {
    const int32_t first = b[sg] > 0 && rows_in(b[sg] - 1, sg) > 0 ? b[sg] - 1 : b[sg];
    tm->seg_key_lo[sg] = seq_lo[first];
  }
  tm->n_d0 = (L + kKeysPerTile - 1) / kKeysPerTile;
  tm->n_csub = K > 1 ? kRowsPerTile / kKeysPerTile : 0;  // a tile's chain keys are rows minus anchors: < 128
  tm->n_key_tiles = tm->n_d0 + tm->n_row_tiles * tm->n_csub;

  // the masks depend on the sample and on where sequences start; equal ones are stored once
  std::vector<uint32_t> bits(kMaskWords);
  std::unordered_map<uint64_t, std::vector<int32_t>> by_hash;
  auto append_mask = [&](const std::vector<uint32_t>& m) {
    uint64_t h = 1469598103934665603ull;
    for (uint32_t w : m) h = (h ^ w) * 1099511628211ull;
    std::vector<int32_t>& ids = by_hash[h];
    for (int32_t id : ids)
      if (std::memcmp(&tm->masks[(size_t)id * kMaskWords], m.data(), kMaskWords * sizeof(uint32_t)) == 0) return id;
    tm->masks.insert(tm->masks.end(), m.begin(), m.end());
    ids.push_back(tm->n_masks);
    return tm->n_masks++;
  };
  std::vector<int32_t> chain_index((size_t)K * kRowsPerTile);  // [depth][anchor - a0] -> index in the tile's chain list
  tm->row_ptr.assign(tm->n_row_tiles + 1, 0);
  tm->row_tok.assign((size_t)tm->n_row_tiles * kRowsPerTile, -1);
  tm->chain_tok.assign((size_t)tm->n_row_tiles * tm->n_csub * kKeysPerTile, -1);
  std::vector<int32_t> row_a(kRowsPerTile), row_d(kRowsPerTile), key_a, key_e;
  for (int32_t R = 0; R < tm->n_row_tiles; ++R) {
    const int32_t a0 = tile_a0[R], a1 = tile_a1[R];
    // rows of the tile, depth-major like the dense tile; chain keys = its rows of depth >= 1
    int rows_used = 0;
    key_a.clear();
    key_e.clear();
    const int32_t sg = tile_seg[R];
    for (int32_t g = 0; g < K; ++g)
      for (int32_t i = a0; i < a1; ++i)
        if (depth_count[i] > g && (g == 0 ? seg_of_pos[i] : chain_seg(i)) == sg) {
          row_a[rows_used] = i;
          row_d[rows_used] = g;
          tm->row_tok[(size_t)R * kRowsPerTile + rows_used] = tok_of[(size_t)g * L + i];
          tm->tok_pos[tok_of[(size_t)g * L + i]] = (int64_t)R * kRowsPerTile + rows_used;
          ++rows_used;
          if (g >= 1) {
            chain_index[(size_t)g * kRowsPerTile + (i - a0)] = (int32_t)key_a.size();
            key_a.push_back(i);
            key_e.push_back(g);
          }
        }
    // depth-0 stream: keys of the tile's own sequence up to its last anchor.  Depth-0 keys are causal
    // in the anchor inside a sequence (sees(i, d, j, 0) == j <= i), so row r sees the keys
    // [sb, row_a[r]] of a tile: a contiguous bit range.  Full tiles are listed first.
    const int32_t sb = seq_lo[a0];
    std::vector<TileEntry> partial_entries;
    std::vector<int32_t> partial_key_ids;
    for (int32_t c = sb / kKeysPerTile; c < tm->n_d0; ++c) {
      const int64_t j0 = (int64_t)c * kKeysPerTile, j1 = j0 + kKeysPerTile - 1;
      if (j0 > a1 - 1) break;
      if (j0 >= sb && j1 <= a0) {
        ++tm->n_full;
        tm->row_entries.push_back(TileEntry{c, -1});
        tm->key_side_id.push_back(-1);
        continue;
      }
      std::fill(bits.begin(), bits.end(), 0u);
      for (int r = 0; r < rows_used; ++r) {
        const int64_t lo = std::max<int64_t>(0, (int64_t)sb - j0);
        const int64_t hi = std::min<int64_t>(kKeysPerTile - 1, (int64_t)row_a[r] - j0);  // inclusive
        if (hi < lo) continue;
        const uint64_t upto_hi = hi >= 63 ? ~0ull : ((1ull << (hi + 1)) - 1);
        const uint64_t m = upto_hi & ~((1ull << lo) - 1);
        bits[r * kMaskWordsPerRow] = (uint32_t)m;
        bits[r * kMaskWordsPerRow + 1] = (uint32_t)(m >> 32);
      }
      partial_entries.push_back(TileEntry{c, append_mask(bits)});
      partial_key_ids.push_back(j1 <= a0 ? -2 - sb : partial_entries.back().mask_id);
      ++tm->n_partial;
    }
    tm->row_entries.insert(tm->row_entries.end(), partial_entries.begin(), partial_entries.end());
    tm->key_side_id.insert(tm->key_side_id.end(), partial_key_ids.begin(), partial_key_ids.end());
    // chain stream
    for (int32_t sub = 0; sub < tm->n_csub; ++sub) {
      const size_t k0 = (size_t)sub * kKeysPerTile;
      if (k0 >= key_a.size()) break;
      std::fill(bits.begin(), bits.end(), 0u);
      const int32_t kt = tm->n_d0 + R * tm->n_csub + sub;
      for (int kk = 0; kk < kKeysPerTile && k0 + kk < key_a.size(); ++kk) {
        const int32_t ja = key_a[k0 + kk], je = key_e[k0 + kk];
        tm->chain_tok[((size_t)R * tm->n_csub + sub) * kKeysPerTile + kk] = tok_of[(size_t)je * L + ja];
      }
      // a chain key (j, e) is seen by the rows of its own anchor at depths >= e (sees(i, d, j, e) ==
      // (j == i && e <= d)): walk each row's own chain instead of testing all pairs
      for (int r = 0; r < rows_used; ++r)
        for (int e = 1; e <= row_d[r]; ++e) {
          const int64_t ck = (int64_t)chain_index[(size_t)e * kRowsPerTile + (row_a[r] - a0)] - (int64_t)k0;
          if (ck >= 0 && ck < kKeysPerTile) bits[r * kMaskWordsPerRow + ck / 32] |= 1u << (ck % 32);
        }
      tm->row_entries.push_back(TileEntry{kt, append_mask(bits)});
      tm->key_side_id.push_back(tm->row_entries.back().mask_id);
      ++tm->n_partial;
    }
    tm->row_ptr[R + 1] = (int32_t)tm->row_entries.size();
    int32_t lead = 0;
    for (int32_t e = tm->row_ptr[R]; e < tm->row_ptr[R + 1] && tm->row_entries[e].mask_id < 0; ++e) ++lead;
    tm->row_lead.push_back(lead);
  }
  return PEAGLE_OK;
}

}  // namespace

// General builder: explicit position set (depth_count, or every depth if null) of a batch of
// sequences packed before the expansion (seq_start, or one sequence if null).
extern "C" int peagle_build_tilemap_packed(const int32_t* depth_count, int32_t L, int32_t K, const int32_t* seq_start,
                                           int32_t n_seq, const int32_t* seg_bounds, int32_t S, int32_t assignment,
                                           int32_t device, peagle_tilemap_t** out) {
  if (!out) return PEAGLE_ENULL;
  *out = nullptr;
  if (device < -1) return PEAGLE_EINVAL;
  peagle_tilemap* tm = new (std::nothrow) peagle_tilemap();
  if (!tm) return PEAGLE_EINVAL;
  const int rc = fill_packed(tm, depth_count, L, K, seq_start, n_seq, seg_bounds, S, assignment);
  if (rc != PEAGLE_OK) {
    delete tm;
    return rc;
  }
  return finish_map(tm, device, out);
}

extern "C" int peagle_tilemap_rebuild(peagle_tilemap_t* tm, const int32_t* depth_count, int32_t L,
                                      const int32_t* seq_start, int32_t n_seq, const int32_t* seg_bounds, int32_t S,
                                      int32_t assignment, void* stream) {
  if (!tm) return PEAGLE_ENULL;
  if (!tm->sampled) return PEAGLE_EUNSUPPORTED;  // the dense map is position-invariant: nothing to rebuild
  const int rc = fill_packed(tm, depth_count, L, tm->K, seq_start, n_seq, seg_bounds, S, assignment);
  if (rc != PEAGLE_OK) return rc;
  build_key_lists(tm);
  return upload_map(tm, (hipStream_t)stream, false);
}

extern "C" int64_t peagle_tilemap_tokens(const peagle_tilemap_t* tm, int32_t L) {
  if (!tm || L < 1 || L > tm->L_max) return -1;
  if (tm->sampled) return L == tm->L_max ? tm->T_tokens : -1;
  return (int64_t)L * tm->K;
}

extern "C" int peagle_tilemap_info(const peagle_tilemap_t* tm, peagle_tilemap_info_t* info) {
  if (!tm || !info) return PEAGLE_ENULL;
  info->L_max = tm->L_max;
  info->K = tm->K;
  info->S = tm->S;
  info->anchors_per_row_tile = tm->A;
  info->rows_per_tile = kRowsPerTile;
  info->keys_per_tile = kKeysPerTile;
  info->n_row_tiles = tm->n_row_tiles;
  info->n_depth0_key_tiles = tm->n_d0;
  info->n_chain_sub_tiles = tm->n_csub;
  info->n_key_tiles = tm->n_key_tiles;
  info->n_full = tm->n_full;
  info->n_partial = tm->n_partial;
  info->n_masks = tm->n_masks;
  info->device_bytes = tm->dev_bytes;
  info->tokens = tm->T_tokens;
  info->sampled = tm->sampled;
  return PEAGLE_OK;
}

int peagle::resolve_segment(const peagle_tilemap* tm, int32_t L, int32_t seg, SegRange* out) {
  if (L < 1 || L > tm->L_max) return PEAGLE_ESHAPE;
  if (seg < -1 || seg >= tm->S) return PEAGLE_EINVAL;
  int32_t lo = 0, hi = L;
  out->s_lo = 0;
  out->s_hi = tm->S;
  if (seg >= 0) {
    lo = tm->seg_bounds[seg];
    hi = tm->seg_bounds[seg + 1] < L ? tm->seg_bounds[seg + 1] : L;
    if (lo > hi) lo = hi;  // segment lies beyond the cropped length: empty
    out->s_lo = seg;
    out->s_hi = seg + 1;
  }
  out->cropped = hi < tm->seg_bounds[out->s_hi];
  out->a_lo = lo;
  out->a_hi = hi;
  out->key_lo = 0;
  if (tm->sampled && seg >= 0) out->key_lo = tm->seg_key_lo[seg];
  if (tm->sampled) {  // built for exactly this sequence: no crop, row tiles from the packing
    if (L != tm->L_max) return PEAGLE_ESHAPE;
    out->rt_lo = tm->seg_rt[out->s_lo];
    out->rt_hi = tm->seg_rt[out->s_hi];
    return PEAGLE_OK;
  }
  out->rt_lo = lo / tm->A;
  out->rt_hi = (hi + tm->A - 1) / tm->A;
  if (lo == hi) out->rt_hi = out->rt_lo;
  return PEAGLE_OK;
}

extern "C" int peagle_tilemap_expand_rows(const peagle_tilemap_t* tm, int32_t L, int32_t seg, int64_t row_begin,
                                          int64_t row_end, uint8_t* bits_out) {
  if (!tm || !bits_out) return PEAGLE_ENULL;
  peagle::SegRange sr;
  int rc = peagle::resolve_segment(tm, L, seg, &sr);
  if (rc != PEAGLE_OK) return rc;
  const int64_t T = tm->sampled ? tm->T_tokens : (int64_t)L * tm->K;
  if (row_begin < 0 || row_end < row_begin || row_end > T) return PEAGLE_EINVAL;
  const int64_t row_bytes = (T + 7) / 8;
  const int A = tm->A;
  const int chain_keys = A * (tm->K - 1);
  std::memset(bits_out, 0, (size_t)((row_end - row_begin) * row_bytes));
  for (int64_t t = row_begin; t < row_end; ++t) {
    int32_t R;
    int r;
    if (tm->sampled) {
      R = (int32_t)(tm->tok_pos[t] / kRowsPerTile);
      r = (int)(tm->tok_pos[t] % kRowsPerTile);
      if (R < sr.rt_lo || R >= sr.rt_hi) continue;
    } else {
      const int64_t i = t % L;
      const int d = (int)(t / L);
      if (i < sr.a_lo || i >= sr.a_hi) continue;
      R = (int32_t)(i / A);
      r = d * A + (int)(i % A);  // row inside the tile
    }
    uint8_t* dst = bits_out + (t - row_begin) * row_bytes;
    for (int32_t e = tm->row_ptr[R]; e < tm->row_ptr[R + 1]; ++e) {
      const TileEntry& en = tm->row_entries[e];
      const uint32_t* mw = en.mask_id < 0 ? nullptr : &tm->masks[(size_t)en.mask_id * kMaskWords + r * kMaskWordsPerRow];
      for (int kk = 0; kk < kKeysPerTile; ++kk) {
        if (mw && !((mw[kk / 32] >> (kk % 32)) & 1u)) continue;
        int64_t tok;
        if (en.tile < tm->n_d0) {
          const int64_t j = (int64_t)en.tile * kKeysPerTile + kk;
          if (j >= L) continue;
          tok = j;
        } else if (tm->sampled) {
          tok = tm->chain_tok[(size_t)(en.tile - tm->n_d0) * kKeysPerTile + kk];
          if (tok < 0) continue;
        } else {
          const int32_t cid = en.tile - tm->n_d0;
          const int ck = (cid % tm->n_csub) * kKeysPerTile + kk;
          if (ck >= chain_keys) continue;
          const int64_t j = (int64_t)(cid / tm->n_csub) * A + ck % A;
          if (j >= L) continue;
          tok = (int64_t)(1 + ck / A) * L + j;
        }
        dst[tok >> 3] |= (uint8_t)(1u << (tok & 7));
      }
    }
  }
  return PEAGLE_OK;
}

extern "C" int peagle_tilemap_classes(const peagle_tilemap_t* tm, uint8_t* classes_out) {
  if (!tm || !classes_out) return PEAGLE_ENULL;
  const size_t n = (size_t)tm->n_row_tiles * tm->n_key_tiles;
  std::memset(classes_out, PEAGLE_TILE_EMPTY, n);
  for (int32_t R = 0; R < tm->n_row_tiles; ++R)
    for (int32_t e = tm->row_ptr[R]; e < tm->row_ptr[R + 1]; ++e) {
      const TileEntry& en = tm->row_entries[e];
      classes_out[(size_t)R * tm->n_key_tiles + en.tile] = en.mask_id < 0 ? PEAGLE_TILE_FULL : PEAGLE_TILE_PARTIAL;
    }
  return PEAGLE_OK;
}

extern "C" const char* peagle_strerror(int status) {
  switch (status) {
    case PEAGLE_OK: return "ok";
    case PEAGLE_EINVAL: return "invalid argument";
    case PEAGLE_ENULL: return "required pointer is NULL";
    case PEAGLE_ESHAPE: return "shape does not fit the tile map (L > L_max or K mismatch)";
    case PEAGLE_EBOUNDS: return "segment bounds must rise strictly from 0 to L_max with inner bounds multiples of 128/K";
    case PEAGLE_EUNSUPPORTED: return "unsupported configuration (head_dim must be 64 or 128, K <= 128, depth-major layout)";
    case PEAGLE_EWORKSPACE: return "workspace missing or too small";
    case PEAGLE_EHIP: return "HIP runtime call failed";
    case PEAGLE_ENODEVICE: return "tile map was built host-only";
    default: return "unknown status";
  }
}
