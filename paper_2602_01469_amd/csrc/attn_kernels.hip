// Block-sparse flash attention forward / backward for the parallel-prediction mask (Sec. 3 of
// the paper), gfx950 only.  Work is organised by the tile map: a row tile is A anchors at all K
// depths (128 rows), key tiles are 64 wide; full pairs skip masking, partial pairs apply a
// bitmask from the pool, empty pairs are never listed.
//
// All score matrices are produced transposed where that keeps the softmax reduction inside a
// lane: in the forward and dQ kernels a lane owns one query row (S^T = K Q^T, lane <-> row,
// registers <-> keys); in the dK/dV kernel a lane owns one key (S = Q K^T, lane <-> key,
// registers <-> rows).  Operands whose contraction index is not contiguous in memory are read
// from LDS with ds_read_b64_tr_b16.
#include "attn_kernels.h"
#include "mfma_util.h"
#include "rope_util.h"

#include <climits>
#include <type_traits>

namespace peagle {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleThreshold = 8.0f;  // log2 units: the running reference max lags by at most 2^8
constexpr float kNegInit = -1.0e30f;
// Bits of a 32-key mask word (already shifted right by 4g) that belong to the keys a lane holds in the
// C layout of a transposed score block: keys 8*(i/4) + 4g + i%4, i = 0..15.
constexpr uint32_t kLaneKeyBits = 0x0f0f0f0fu;

// Token (row of the [T, H, D] tensors) of key `row` of key tile `kt`; false if that key does not
// exist in a length-L problem.
__device__ __forceinline__ bool key_token(const DeviceTileMap& tm, int kt, int row, int L, int& tok) {
  if (kt < tm.n_d0) {
    tok = kt * kKeysPerTile + row;
    return tok < L;
  }
  const int cid = kt - tm.n_d0;
  if (tm.row_tok) {  // sampled map: explicit list of the tile's chain keys
    tok = tm.chain_tok[(size_t)cid * kKeysPerTile + row];
    return tok >= 0;
  }
  const int R = cid / tm.n_csub;
  const int ck = (cid - R * tm.n_csub) * kKeysPerTile + row;
  const int e = ck / tm.A;
  const int j = R * tm.A + (ck - e * tm.A);
  tok = (1 + e) * L + j;
  return ck < tm.A * (tm.K - 1) && j < L;
}

// Token of row `r` of row tile `rt`; false if the row is padding or beyond the sequence.
__device__ __forceinline__ bool row_token(const DeviceTileMap& tm, int rt, int r, int L, int& tok) {
  if (tm.row_tok) {  // sampled map: explicit list of the tile's rows
    tok = tm.row_tok[(size_t)rt * kRowsPerTile + r];
    return tok >= 0;
  }
  const int d = r / tm.A;
  const int i = rt * tm.A + (r - d * tm.A);
  tok = d * L + i;
  return d < tm.K && i < L;
}

__device__ __forceinline__ uint4 ld16(const __bf16* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ bf16x8 as_frag(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// Entry `e` of a tile list, made wave-uniform (the index is uniform; this lets branches on the
// entry be scalar).  Lists are read two iterations ahead of their use: fetch_entry() starts the
// load early in an iteration, take_entry() - called after the iteration's barrier - moves the
// value to scalar registers.  The empty assembly statement pins that move below the barrier;
// without it the compiler places it, and the wait for the load, right behind the load.
__device__ __forceinline__ u32x2 fetch_entry(const TileEntry* list, int e) {
  return *reinterpret_cast<const u32x2*>(list + e);
}
__device__ __forceinline__ TileEntry take_entry(u32x2 w) {
  uint32_t w0 = w[0], w1 = w[1];
  asm volatile("" : "+v"(w0), "+v"(w1) : : "memory");
  TileEntry en;
  en.tile = __builtin_amdgcn_readfirstlane((int)w0);
  en.mask_id = __builtin_amdgcn_readfirstlane((int)w1);
  return en;
}
__device__ __forceinline__ TileEntry load_entry(const TileEntry* list, int e) { return take_entry(fetch_entry(list, e)); }

// LDS addresses of the K/V tile buffers of the row-stationary kernels, [slot][K|V][tile bytes], as plain scalar
// integers: the address of slot 0 is taken once per kernel and everything else is integer arithmetic (taken
// per copy from a pointer, each address costs a null check and two moves to the scalar unit).
template <int D>
struct KeyTileLds {
  uint32_t base;  // address of slot 0's K image + 1024 * wave
  __device__ __forceinline__ KeyTileLds(const char* slot0, int wave)
      : base(lds_scalar_addr(slot0 + wave * 1024)) {}
  __device__ __forceinline__ uint32_t k(int slot) const { return base + (uint32_t)slot * (2u * kKeysPerTile * D * 2); }
  __device__ __forceinline__ uint32_t v(int slot) const { return k(slot) + kKeysPerTile * D * 2; }
};

// Key tile straight into its swizzled LDS image (K and V): wave w of NW fills the 1 KiB blocks
// w, w + NW, ...; lane l of block b owns LDS bytes [1024 b + 16 l, +16), i.e. tile row
// b*(512/D) + l/(D/8) and physical chunk l%(D/8), and fetches the logical chunk that lives there.
template <int D, int NW, bool SV = false>
__device__ __forceinline__ void dma_key_tile(uint32_t kd, uint32_t vd, const __bf16* kbase, const __bf16* vbase,
                                             int Hkv, int kvh, const DeviceTileMap& tm, int kt, int L, int wave,
                                             int lane, const __bf16* v_shared = nullptr) {
  // kd, vd: LDS byte addresses of this wave's first block of the K and of the V image (tile address + 1024 *
  // wave), as wave-uniform integers - see KeyTileLds
  constexpr int kBlocks = kKeysPerTile * D * 2 / 1024;
  static_assert(kBlocks % NW == 0, "tile must split evenly over the waves");
  const int row_in_blk = lane / (D / 8), phys = lane % (D / 8);
  if (kt < tm.n_d0 && (kt + 1) * kKeysPerTile <= L) {
    // A whole tile of depth-0 keys: the rows a lane copies are NW * 512/D apart (a multiple of the swizzle
    // period), so its byte offset from each copy's first row is one value, the same for every tile, and the
    // rest of the address is wave-uniform.
    const int row0 = wave * (512 / D) + row_in_blk;
    const uint32_t voff = (uint32_t)((row0 * Hkv) * D + ((phys ^ swz<D>(row0)) << 3)) * 2u;
#pragma unroll
    for (int i = 0; i < kBlocks / NW; ++i) {
      const size_t first = ((size_t)(kt * kKeysPerTile + i * NW * (512 / D)) * Hkv + kvh) * D;
      dma16_untracked(uniform_ptr(kbase + first), voff, kd + i * NW * 1024);
      dma16_untracked(uniform_ptr(vbase + first), voff, vd + i * NW * 1024);
    }
  } else if (SV && kt >= tm.n_d0) {
    // First-layer form, chain tile: every key's value row is the one shared vector of its KV head.  (SV is a
    // template flag: kernels of the ordinary step carry none of this.)
#pragma unroll
    for (int i = 0; i < kBlocks / NW; ++i) {
      const int blk = i * NW + wave;
      const int row = blk * (512 / D) + row_in_blk;
      int tok;
      const bool ok = key_token(tm, kt, row, L, tok);
      const int chunk = (phys ^ swz<D>(row)) << 3;
      const size_t off = ((size_t)(ok ? tok : 0) * Hkv + kvh) * D + chunk;
      dma16_untracked(ok ? (const void*)(kbase + off) : tm.zeros, kd + i * NW * 1024);
      dma16_untracked(ok ? (const void*)(v_shared + (size_t)kvh * D + chunk) : tm.zeros, vd + i * NW * 1024);
    }
  } else {
#pragma unroll
    for (int i = 0; i < kBlocks / NW; ++i) {
      const int blk = i * NW + wave;
      const int row = blk * (512 / D) + row_in_blk;
      int tok;
      const bool ok = key_token(tm, kt, row, L, tok);
      const size_t off = ((size_t)(ok ? tok : 0) * Hkv + kvh) * D + ((phys ^ swz<D>(row)) << 3);
      dma16_untracked(ok ? (const void*)(kbase + off) : tm.zeros, kd + i * NW * 1024);
      dma16_untracked(ok ? (const void*)(vbase + off) : tm.zeros, vd + i * NW * 1024);
    }
  }
}

// Row tile (128 rows of one query head) straight into its swizzled LDS image, same block/lane
// assignment as dma_key_tile; rows that do not exist are filled from the zero page.  The rows a
// lane copies are the same for every row tile, so their (depth, anchor) split - which costs an
// integer division by A - is done once per kernel (RowDmaLane) and a copy only adds rt*A.
template <int D, int NW>
struct RowDmaLane {
  static constexpr int kBlocks = kRowsPerTile * D * 2 / 1024;
  static constexpr int kPer = kBlocks / NW;
  static_assert(kBlocks % NW == 0, "tile must split evenly over the waves");
  int tok0[kPer];    // d*L + a : token of the row in row tile 0 (dense map)
  int a[kPer];       // anchor offset inside the row tile; >= A*K... marks a padding row via a huge value
  int row[kPer];     // row of the tile (index into a sampled map's row list)
  int chunk[kPer];   // element offset of the logical 16-byte chunk this lane fetches
  int stat_tok0, stat_a, stat_row;  // same for the row whose per-row statistic this lane copies (waves 0..3)
  // Dense maps, row tiles whose 128 rows all exist: byte offset of each copy's source from the head's row of the
  // tile's first anchor, ((d*L + a) * Hq) * D * 2 + 2 * chunk (and 4 * (d*L + a) for the statistic) - the same
  // for every row tile and head, so a copy needs only a new scalar base.
  uint32_t fast_off[kPer], fast_stat_off;
};
template <int D, int NW>
__device__ __forceinline__ RowDmaLane<D, NW> row_dma_lane(const DeviceTileMap& tm, int L, int wave, int lane, int Hq = 0) {
  RowDmaLane<D, NW> r;
  const int row_in_blk = lane / (D / 8), phys = lane % (D / 8);
#pragma unroll
  for (int i = 0; i < RowDmaLane<D, NW>::kPer; ++i) {
    const int row = (i * NW + wave) * (512 / D) + row_in_blk;
    const int A = tm.row_tok ? 1 : tm.A;  // a sampled map has no fixed geometry; rows come from its list
    const int d = row / A, a = row - d * A;
    r.tok0[i] = d * L + a;
    r.a[i] = d < tm.K ? a : (1 << 30);
    r.row[i] = row;
    r.chunk[i] = (phys ^ swz<D>(row)) << 3;
    r.fast_off[i] = (uint32_t)r.tok0[i] * (uint32_t)(Hq * D * 2) + (uint32_t)(r.chunk[i] * 2);
  }
  const int srow = (wave & 1) * 64 + lane;
  const int A = tm.row_tok ? 1 : tm.A;
  const int sd = srow / A, sa = srow - sd * A;
  r.stat_tok0 = sd * L + sa;
  r.stat_a = sd < tm.K ? sa : (1 << 30);
  r.stat_row = srow;
  r.fast_stat_off = (uint32_t)r.stat_tok0 * 4u;
  return r;
}
// Tokens of the rows this lane copies for one row tile (-1: the row does not exist).  For a dense map
// they are arithmetic; a sampled / packed map lists them, and the loads are issued an iteration
// before the copy that needs them so that their latency does not add to the copy's.
template <int D, int NW>
struct RowTokens {
  int tok[RowDmaLane<D, NW>::kPer];
  int stat_tok;
};
template <int D, int NW, bool LISTED>
__device__ __forceinline__ RowTokens<D, NW> row_tokens(const DeviceTileMap& tm, const RowDmaLane<D, NW>& rl, int rt,
                                                       int L) {
  RowTokens<D, NW> t;
  if (LISTED) {
    const int32_t* list = tm.row_tok + (size_t)rt * kRowsPerTile;
#pragma unroll
    for (int i = 0; i < RowDmaLane<D, NW>::kPer; ++i) t.tok[i] = list[rl.row[i]];
    t.stat_tok = list[rl.stat_row];
  } else {
    const int i0 = rt * tm.A;
#pragma unroll
    for (int i = 0; i < RowDmaLane<D, NW>::kPer; ++i) t.tok[i] = i0 + rl.a[i] < L ? rl.tok0[i] + i0 : -1;  // padding rows carry a huge anchor offset
    t.stat_tok = i0 + rl.stat_a < L ? rl.stat_tok0 + i0 : -1;
  }
  return t;
}
template <int D, int NW>
__device__ __forceinline__ void dma_row_tile(char* lds_tile, const __bf16* base, int Hq, int h, const DeviceTileMap& tm,
                                             const RowDmaLane<D, NW>& rl, const RowTokens<D, NW>& t, int wave) {
  const uint32_t dst = lds_scalar_addr(lds_tile + wave * 1024);
#pragma unroll
  for (int i = 0; i < RowDmaLane<D, NW>::kPer; ++i) {
    const bool ok = t.tok[i] >= 0;
    const size_t off = ((size_t)(ok ? t.tok[i] : 0) * Hq + h) * D + rl.chunk[i];
    dma16_untracked(ok ? (const void*)(base + off) : tm.zeros, dst + i * NW * 1024);
  }
}

// Per-row fp32 statistic of a row tile (128 values, [Hq, T] array) into LDS: two waves of the
// caller each fill 64 rows (half = wave & 1).
template <int D, int NW>
__device__ __forceinline__ void dma_row_stat(float* lds_stat, const float* base, int T, int h, const DeviceTileMap& tm,
                                             const RowTokens<D, NW>& t, int half) {
  const bool ok = t.stat_tok >= 0;
  dma4_untracked(ok ? (const void*)(base + (size_t)h * T + t.stat_tok) : tm.zeros,
                 lds_scalar_addr(reinterpret_cast<const char*>(lds_stat + half * 64)));
}

// Does any row of the wave see a key of the 32-key block whose (shifted) mask word each lane holds?
__device__ __forceinline__ bool wave_sees_block(uint32_t mw) {
  return __builtin_amdgcn_ballot_w64((mw & kLaneKeyBits) != 0) != 0;
}

// Bit `pos` of w selects x, otherwise -inf.
__device__ __forceinline__ float mask_sel(float x, uint32_t w, int pos) {
  return ((w >> pos) & 1u) ? x : -__builtin_inff();
}

__device__ __forceinline__ float max16(const f32x16& s) {
  float a = __builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), s[2]);
  float b = __builtin_fmaxf(__builtin_fmaxf(s[3], s[4]), s[5]);
  float c = __builtin_fmaxf(__builtin_fmaxf(s[6], s[7]), s[8]);
  float d = __builtin_fmaxf(__builtin_fmaxf(s[9], s[10]), s[11]);
  float e = __builtin_fmaxf(__builtin_fmaxf(s[12], s[13]), s[14]);
  a = __builtin_fmaxf(__builtin_fmaxf(a, b), c);
  d = __builtin_fmaxf(__builtin_fmaxf(d, e), s[15]);
  return __builtin_fmaxf(a, d);
}

// Online-softmax update for one 32-key block of one head.  On entry s holds raw q.k of the
// lane's row for its 16 keys; on exit pb holds exp2(s*c - m) as two bf16 B-operand fragments.
// The reference max m moves only when the block exceeds it by more than the threshold, which
// keeps the accumulator rescale off the common path without affecting the result.
template <int DB, bool MASKED>
__device__ __forceinline__ void softmax_block(f32x16& s, uint32_t mw, float c, float& m, float& lsum,
                                              f32x16 (&o)[DB], bf16x8 (&pb)[2]) {
  if (MASKED) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = mask_sel(s[i], mw, 8 * (i / 4) + (i % 4));
  }
  const float mx = max_halves(max16(s)) * c;
  const bool need = mx > m + kRescaleThreshold;
  if (__builtin_amdgcn_ballot_w64(need) != 0) {
    const float m_new = need ? mx : m;
    const float alpha = exp2_fast(m - m_new);
    m = m_new;
    lsum *= alpha;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
  }
  const float neg_m = -m;
#pragma unroll
  for (int i = 0; i < 16; ++i) s[i] = exp2_fast(__builtin_fmaf(s[i], c, neg_m));
  pb[0] = pack8_sum(s, 0, lsum);
  pb[1] = pack8_sum(s, 1, lsum);
}

}  // namespace

// =====================================================================================
// Forward: O = softmax(scale Q K^T + mask) V, LSE.  One workgroup (4 waves) per
// (row tile, NH query heads of one KV group); wave w owns rows [32w, 32w+32) of the tile.
// K/V tiles are staged once in LDS per workgroup and serve all NH heads.
// =====================================================================================
template <int D, int NH, bool MASKED, bool SAFE>
__device__ __forceinline__ void fwd_tile(const char* kt_lds, const char* vt_lds, const NatOff<D>& no, const TrOff<D>& to,
                                         const bf16x8 (&qf)[NH][D / 16], f32x16 (&o)[NH][D / 32], float (&m)[NH],
                                         float (&lsum)[NH], const uint32_t (&mw)[2], float c) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {  // the tile's two 32-key blocks
    // S^T block: 32 keys x 32 rows, lane <-> row, registers <-> keys 8*(i/4) + 4g + i%4
    f32x16 s[NH];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) s[hh] = zero16();
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const bf16x8 a = frag_nat<D>(kt_lds, no, kb, st);
#pragma unroll
      for (int hh = 0; hh < NH; ++hh) s[hh] = mfma32(a, qf[hh][st], s[hh]);
    }
    bf16x8 pb[NH][2];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      if (SAFE) {
        softmax_block<D / 32, MASKED>(s[hh], mw[kb], c, m[hh], lsum[hh], o[hh], pb[hh]);
      } else {  // reference max fixed at 0: p = 2^(c s); the caller checks the row sums' range
        if (MASKED) {
#pragma unroll
          for (int i = 0; i < 16; ++i) s[hh][i] = mask_sel(s[hh][i], mw[kb], 8 * (i / 4) + (i % 4));
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) s[hh][i] = exp2_fast(s[hh][i] * c);
        pb[hh][0] = pack8_sum(s[hh], 0, lsum[hh]);
        pb[hh][1] = pack8_sum(s[hh], 1, lsum[hh]);
      }
    }
    // O^T += V^T P^T : A = V^T (lane <-> d, contraction over the block's 32 keys)
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 a = frag_tr<D>(vt_lds, to, kb * 32 + t * 16, db);
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) o[hh][db] = mfma32(a, pb[hh][t], o[hh][db]);
      }
  }
}

template <int D, int NH, bool SV>
__global__ __launch_bounds__(256, 2) void fwd_kernel(FwdParams p) {
  constexpr int kTileBytes = kKeysPerTile * D * 2;
  __shared__ __attribute__((aligned(16))) char lds[2][2][kTileBytes];  // [buffer][K|V]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const KeyTileLds<D> kl(&lds[0][0][0], wave);
  const DeviceTileMap& tm = p.tm;
  const int group = p.Hq / p.Hkv;
  const int hpg = group / NH;
  int b = blockIdx.x;
  const int kvh = b % p.Hkv;
  b /= p.Hkv;
  const int hc = b % hpg;
  const int rt = p.rt_hi - 1 - b / hpg;  // heaviest row tiles first
  const int h0 = kvh * group + hc * NH;

  const int r = wave * 32 + ln;  // row of the tile owned by this lane (shared with lane^32)
  int tq;
  const bool row_ok = row_token(tm, rt, r, p.L, tq);

  bf16x8 qf[NH][D / 16];
#pragma unroll
  for (int hh = 0; hh < NH; ++hh)
#pragma unroll
    for (int st = 0; st < D / 16; ++st)
      qf[hh][st] = as_frag(row_ok ? ld16(p.q + ((size_t)tq * p.Hq + h0 + hh) * D + st * 16 + g * 8)
                                  : make_uint4(0, 0, 0, 0));

  f32x16 o[NH][D / 32];
  float m[NH], lsum[NH], l_tot[NH];
  const NatOff<D> no = nat_offsets<D>(lane);
  const TrOff<D> to = tr_offsets<D>(lane);
  const int e0 = tm.row_ptr[rt], e1 = tm.row_ptr[rt + 1];
  const int e_lead = e0 + tm.row_lead[rt];  // end of the leading run of full tiles

  // One pass over the row tile's key tiles.  The first pass keeps the softmax reference at 0
  // (no running max: fewer vector instructions per score); it is exact as long as every row
  // sum stays inside the fp32 / bf16 exponent range.  If any row of the workgroup leaves
  // [2^-100, 2^100] (or is not finite) the tile is recomputed with the running-max form.
  auto pass = [&](auto safe_tag) {
    constexpr bool SAFE = decltype(safe_tag)::value;
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      m[hh] = SAFE ? kNegInit : 0.f;
      lsum[hh] = 0.f;
#pragma unroll
      for (int db = 0; db < D / 32; ++db) o[hh][db] = zero16();
    }
    TileEntry cur = load_entry(tm.row_entries, e0);
    TileEntry nxt = load_entry(tm.row_entries, e0 + 1 < e1 ? e0 + 1 : e0);
    dma_key_tile<D, 4, SV>(kl.k(0), kl.v(0), p.k, p.v, p.Hkv, kvh, tm, cur.tile, p.L, wave, lane, p.v_shared);
    dma_publish();
    // The leading full tiles run in a counted loop of their own (no mask branch, accumulators
    // stay in place); the partial tiles that end a row tile's list take the general loop.
    int e = e0;
    auto full_tile = [&](int buf) {
      const u32x2 ahead = fetch_entry(tm.row_entries, e + 2 < e1 ? e + 2 : e);
      if (e + 1 < e1)
        dma_key_tile<D, 4, SV>(kl.k(buf ^ 1), kl.v(buf ^ 1), p.k, p.v, p.Hkv, kvh, tm, nxt.tile, p.L, wave, lane, p.v_shared);
      const uint32_t mw[2] = {0xffffffffu, 0xffffffffu};
      fwd_tile<D, NH, false, SAFE>(lds[buf][0], lds[buf][1], no, to, qf, o, m, lsum, mw, p.c_log2);
      dma_publish();
      cur = nxt;
      nxt = take_entry(ahead);
      ++e;
    };
    // (two at a time with the buffer index a constant: every LDS address is then a per-lane register plus an
    // immediate, which saves the eight vector additions per tile that a buffer index in a register costs)
    while (e + 1 < e_lead) {
      full_tile(0);
      full_tile(1);
    }
    if (e < e_lead) full_tile(0);
    for (; e < e1; ++e) {
      const int buf = (e - e0) & 1;
      const u32x2 ahead = fetch_entry(tm.row_entries, e + 2 < e1 ? e + 2 : e);
      if (e + 1 < e1)
        dma_key_tile<D, 4, SV>(kl.k(buf ^ 1), kl.v(buf ^ 1), p.k, p.v, p.Hkv, kvh, tm, nxt.tile, p.L, wave, lane, p.v_shared);
      if (cur.mask_id < 0) {
        const uint32_t mw[2] = {0xffffffffu, 0xffffffffu};
        fwd_tile<D, NH, false, SAFE>(lds[buf][0], lds[buf][1], no, to, qf, o, m, lsum, mw, p.c_log2);
      } else {
        const u32x2 w = *reinterpret_cast<const u32x2*>(tm.masks + ((size_t)cur.mask_id * kRowsPerTile + r) * 2);
        const uint32_t mw[2] = {w[0] >> (4 * g), w[1] >> (4 * g)};
        fwd_tile<D, NH, true, SAFE>(lds[buf][0], lds[buf][1], no, to, qf, o, m, lsum, mw, p.c_log2);
      }
      dma_publish();
      cur = nxt;
      nxt = take_entry(ahead);
    }
    bool bad = false;
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      l_tot[hh] = sum_halves(lsum[hh]);
      bad |= !(l_tot[hh] > 0x1p-100f && l_tot[hh] < 0x1p100f);
    }
    return bad && row_ok;
  };
  if (__syncthreads_or(pass(std::false_type{}))) (void)pass(std::true_type{});

#pragma unroll
  for (int hh = 0; hh < NH; ++hh) {
    const float inv = 1.0f / l_tot[hh];
    if (row_ok) {
      __bf16* orow = p.o + ((size_t)tq * p.Hq + h0 + hh) * D;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(o[hh][db][4 * q4 + 0] * inv, o[hh][db][4 * q4 + 1] * inv);
          w[1] = pack_bf16(o[hh][db][4 * q4 + 2] * inv, o[hh][db][4 * q4 + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + db * 32 + 8 * q4 + 4 * g) = w;
        }
      if (g == 0) p.lse[(size_t)(h0 + hh) * p.T + tq] = (m[hh] + __builtin_log2f(l_tot[hh])) * kLn2;
    }
  }
}

// =====================================================================================
// Backward, part 1: Delta = rowsum(dO * O) and dQ = scale * dS K, row-tile owned (same
// decomposition as the forward).  Writes Delta [Hq, T] for part 2.
// =====================================================================================
template <int D, int NH, bool MASKED, int KB0 = 0, int KB1 = 2>
__device__ __forceinline__ void dq_tile(const char* kt_lds, const char* vt_lds, const NatOff<D>& no, const TrOff<D>& to,
                                        const bf16x8 (&qf)[NH][D / 16], const bf16x8 (&dof)[NH][D / 16],
                                        f32x16 (&dq)[NH][D / 32], const float (&lse2)[NH], const float (&delta)[NH],
                                        const uint32_t (&mw)[2], float c) {
#pragma unroll
  for (int kb = KB0; kb < KB1; ++kb) {
    f32x16 s[NH], dp[NH];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      s[hh] = zero16();
      dp[hh] = zero16();
    }
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const bf16x8 ak = frag_nat<D>(kt_lds, no, kb, st);
      const bf16x8 av = frag_nat<D>(vt_lds, no, kb, st);
#pragma unroll
      for (int hh = 0; hh < NH; ++hh) {
        s[hh] = mfma32(ak, qf[hh][st], s[hh]);     // S^T  = K Q^T
        dp[hh] = mfma32(av, dof[hh][st], dp[hh]);  // dP^T = V dO^T
      }
    }
    bf16x8 dsb[NH][2];
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      if (MASKED) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[hh][i] = mask_sel(s[hh][i], mw[kb], 8 * (i / 4) + (i % 4));
      }
      const float nl = -lse2[hh], dl = delta[hh];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pr = exp2_fast(__builtin_fmaf(s[hh][i], c, nl));
        s[hh][i] = pr * (dp[hh][i] - dl);
      }
      dsb[hh][0] = pack8(s[hh], 0);
      dsb[hh][1] = pack8(s[hh], 1);
    }
    // dQ^T += K^T dS^T : A = K^T (lane <-> d, contraction over the block's keys)
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 a = frag_tr<D>(kt_lds, to, kb * 32 + t * 16, db);
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) dq[hh][db] = mfma32(a, dsb[hh][t], dq[hh][db]);
      }
  }
}

// (This plain form serves D = 128, one query head per workgroup; D = 64 runs dq_pipe_kernel below.  NH stays a
// named constant because dq_tile is written for NH heads sharing the K / V fragments.)
template <int D>
__global__ __launch_bounds__(256, 2) void dq_kernel(BwdParams p) {
  constexpr int NH = 1;
  constexpr int kTileBytes = kKeysPerTile * D * 2;
  __shared__ __attribute__((aligned(16))) char lds[2][2][kTileBytes];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const DeviceTileMap& tm = p.tm;
  const int group = p.Hq / p.Hkv;
  const int hpg = group / NH;
  int b = blockIdx.x;
  const int kvh = b % p.Hkv;
  b /= p.Hkv;
  const int hc = b % hpg;
  const int rt = p.rt_hi - 1 - b / hpg;
  const int h0 = kvh * group + hc * NH;

  const int r = wave * 32 + ln;
  int tq;
  const bool row_ok = row_token(tm, rt, r, p.L, tq);

  bf16x8 qf[NH][D / 16], dof[NH][D / 16];
  float lse2[NH], delta[NH];
#pragma unroll
  for (int hh = 0; hh < NH; ++hh) {
    const size_t off = ((size_t)(row_ok ? tq : 0) * p.Hq + h0 + hh) * D + g * 8;
    float dl = 0.f;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const uint4 z = make_uint4(0, 0, 0, 0);
      qf[hh][st] = as_frag(row_ok ? ld16(p.q + off + st * 16) : z);
      dof[hh][st] = as_frag(row_ok ? ld16(p.d_o + off + st * 16) : z);
      const bf16x8 of = as_frag(row_ok ? ld16(p.o + off + st * 16) : z);
#pragma unroll
      for (int j = 0; j < 8; ++j) dl = __builtin_fmaf((float)dof[hh][st][j], (float)of[j], dl);
    }
    dl = sum_halves(dl);
    delta[hh] = dl;
    lse2[hh] = row_ok ? p.lse[(size_t)(h0 + hh) * p.T + tq] * kLog2e : 0.f;
    if (row_ok && g == 0) {  // per-row terms in the form the dK/dV kernel consumes
      p.delta[(size_t)(h0 + hh) * p.T + tq] = -dl;
      p.nlse[(size_t)(h0 + hh) * p.T + tq] = -lse2[hh] / p.c_log2;
    }
  }

  f32x16 dq[NH][D / 32];
#pragma unroll
  for (int hh = 0; hh < NH; ++hh)
#pragma unroll
    for (int db = 0; db < D / 32; ++db) dq[hh][db] = zero16();

  const NatOff<D> no = nat_offsets<D>(lane);
  const TrOff<D> to = tr_offsets<D>(lane);
  const int e0 = tm.row_ptr[rt], e1 = tm.row_ptr[rt + 1];
  const int e_lead = e0 + tm.row_lead[rt];  // end of the leading run of full tiles
  TileEntry cur = load_entry(tm.row_entries, e0);
  TileEntry nxt = load_entry(tm.row_entries, e0 + 1 < e1 ? e0 + 1 : e0);
  // (LDS addresses taken per copy from the buffers' pointers here, not through KeyTileLds: this kernel is at
  // the register limit, and with the integer form the allocator spilled 96 registers instead
  // of 37 and the kernel ran 7 % slower)
  dma_key_tile<D, 4>(lds_scalar_addr(lds[0][0] + wave * 1024), lds_scalar_addr(lds[0][1] + wave * 1024), p.k, p.v, p.Hkv, kvh, tm, cur.tile, p.L, wave, lane);
  dma_publish();

  int e = e0;
  for (; e < e_lead; ++e) {  // leading full tiles: counted loop, no mask branch
    const int buf = (e - e0) & 1;
    const u32x2 ahead = fetch_entry(tm.row_entries, e + 2 < e1 ? e + 2 : e);
    if (e + 1 < e1)
      dma_key_tile<D, 4>(lds_scalar_addr(lds[buf ^ 1][0] + wave * 1024), lds_scalar_addr(lds[buf ^ 1][1] + wave * 1024), p.k, p.v, p.Hkv, kvh, tm, nxt.tile, p.L, wave, lane);
    const uint32_t mw[2] = {0xffffffffu, 0xffffffffu};
    dq_tile<D, NH, false>(lds[buf][0], lds[buf][1], no, to, qf, dof, dq, lse2, delta, mw, p.c_log2);
    dma_publish();
    cur = nxt;
    nxt = take_entry(ahead);
  }
  for (; e < e1; ++e) {
    const int buf = (e - e0) & 1;
    const u32x2 ahead = fetch_entry(tm.row_entries, e + 2 < e1 ? e + 2 : e);
    if (e + 1 < e1)
      dma_key_tile<D, 4>(lds_scalar_addr(lds[buf ^ 1][0] + wave * 1024), lds_scalar_addr(lds[buf ^ 1][1] + wave * 1024), p.k, p.v, p.Hkv, kvh, tm, nxt.tile, p.L, wave, lane);
    if (cur.mask_id < 0) {
      const uint32_t mw[2] = {0xffffffffu, 0xffffffffu};
      dq_tile<D, NH, false>(lds[buf][0], lds[buf][1], no, to, qf, dof, dq, lse2, delta, mw, p.c_log2);
    } else {
      const u32x2 w = *reinterpret_cast<const u32x2*>(tm.masks + ((size_t)cur.mask_id * kRowsPerTile + r) * 2);
      const uint32_t mw[2] = {w[0] >> (4 * g), w[1] >> (4 * g)};
      // A 32-key block that none of the wave's 32 rows can see contributes exact zeros and is left out:
      // half of a row tile's chain keys are deeper than a given wave's rows, and the second half of a
      // diagonal depth-0 tile is often in the future of the whole row tile.
      // (The forward does not do this: at two heads per workgroup it has no registers to spare, and a
      // second code path there spills.)
      const bool see0 = wave_sees_block(mw[0]), see1 = wave_sees_block(mw[1]);
      if (see0 && see1) dq_tile<D, NH, true>(lds[buf][0], lds[buf][1], no, to, qf, dof, dq, lse2, delta, mw, p.c_log2);
      else if (see0) dq_tile<D, NH, true, 0, 1>(lds[buf][0], lds[buf][1], no, to, qf, dof, dq, lse2, delta, mw, p.c_log2);
      else if (see1) dq_tile<D, NH, true, 1, 2>(lds[buf][0], lds[buf][1], no, to, qf, dof, dq, lse2, delta, mw, p.c_log2);
    }
    dma_publish();
    cur = nxt;
    nxt = take_entry(ahead);
  }

  if (row_ok) {
    if (p.rope_table) {
      // q was the rotated copy: turn dQ back.  The lane holds features db*32 + 8*q4 + 4g + j of its
      // row, so both members of every pair (feature, feature + D/2) are in its own registers.
      const float* rope = p.rope_table + (size_t)token_position(tm, tq, p.L) * D;
#pragma unroll
      for (int db = 0; db < D / 64; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = db * 32 + 8 * q4 + 4 * g;
          const f32x4 cs = *reinterpret_cast<const f32x4*>(rope + d0);
          const f32x4 sn = *reinterpret_cast<const f32x4*>(rope + D / 2 + d0);
#pragma unroll
          for (int hh = 0; hh < NH; ++hh) {
            f32x4 lo, hi;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              lo[j] = dq[hh][db][4 * q4 + j];
              hi[j] = dq[hh][db + D / 64][4 * q4 + j];
            }
            rope_turn4<true>(lo, hi, cs, sn);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              dq[hh][db][4 * q4 + j] = lo[j];
              dq[hh][db + D / 64][4 * q4 + j] = hi[j];
            }
          }
        }
    }
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      __bf16* drow = p.dq + ((size_t)tq * p.Hq + h0 + hh) * D;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(dq[hh][db][4 * q4 + 0] * p.scale, dq[hh][db][4 * q4 + 1] * p.scale);
          w[1] = pack_bf16(dq[hh][db][4 * q4 + 2] * p.scale, dq[hh][db][4 * q4 + 3] * p.scale);
          *reinterpret_cast<u32x2*>(drow + db * 32 + 8 * q4 + 4 * g) = w;
        }
    }
  }
}

// =====================================================================================
// Backward, part 1 with the leading full tiles of a row tile run as one software pipeline (D = 64; same
// decomposition and results layout as dq_kernel).  The unit of work is a 32-key block, two per key tile.
// A wave that issues a matrix instruction and then independent vector instructions runs the vector work
// in the shadow of the matrix pipe, whereas matrix and vector phases that follow one another - in one wave
// or in several waves of a SIMD - take the sum of their times (see dkdv_rowtile_pipelined).  So while the
// vector unit turns the scores of unit u into dS, the matrix pipe runs dQ += K^T dS of unit u-1 and S, dP
// of unit u+1, across key-tile boundaries: three K/V buffers rotate (tile e of the row tile's list lives in
// buffer e % 3; the pipelined tiles are taken three at a time so that every LDS address is a per-lane
// register plus an immediate), the copy of tile e+2 is issued when every wave has left tile e-1, and one
// barrier per tile - between its two units - both frees that buffer and publishes tile e+1.
//
// Per-row terms cost no vector instruction here: -Delta is the accumulator input of the first dP
// instruction (sixteen equal registers per lane, lane <-> row), and the probabilities are left
// unnormalised, p' = 2^(c s), the factor 2^(-lse) being applied to the row's dQ once at the end.  That is
// exact as long as 2^(c s) cannot leave the fp32 range, which |lse| <= 64 (log2 units) guarantees for
// every key of the row; a workgroup with a row outside that range (or a non-finite lse) takes the plain
// routine with the normalised probabilities for all its tiles.
// Tiles that carry a bitmask (the diagonal and chain tiles that end a row tile's list) and the up to two
// full tiles left over by the groups of three go through dq_tile, in the same buffers.
// =====================================================================================
constexpr int kDqAhead = 2;

template <int D>
struct DqPipe {
  f32x16 sc[2], dpc[2];     // S and dP of the units in flight (index = 32-key block of the unit's tile)
  u32x4 dsb[2][2];          // dS of a unit as bf16 B operands, per 16-key step
  bf16x8 ring[kDqAhead];    // A operands on their way from LDS
};

// A operand of matrix instruction j of a unit's body: first the D/16 transposed K fragments of the unit whose
// dQ is due (j = 16-key step * D/32 + feature block), then the D/8 natural fragments of the unit whose S / dP
// start (even: K, odd: V).
template <int D>
__device__ __forceinline__ bf16x8 dq_pipe_frag(const char* k_dq, int kb_dq, const char* k_s, const char* v_s, int kb_s,
                                               const NatOff<D>& no, const TrOff<D>& to, int j) {
  constexpr int N2 = D / 16;
  if (j < N2) return frag_tr<D>(k_dq, to, kb_dq * 32 + (j / (D / 32)) * 16, j % (D / 32));
  const int i = j - N2;
  return frag_nat<D>((i & 1) ? v_s : k_s, no, kb_s, i >> 1);
}

// Body of the unit (tile e, block KB): its vector work rides on the matrix instructions dQ of the unit before
// it (block 1-KB of k_dq: tile e-1 for KB = 0, tile e for KB = 1) and, unless LAST, S / dP of the unit after it
// (block 1-KB of k_s, v_s: tile e for KB = 0, tile e+1 for KB = 1).  k_self is K of tile e: the next body's
// dQ fragments (this unit's) are prefetched from it.
template <int D, int KB, bool LAST>
__device__ __forceinline__ void dq_pipe_body(DqPipe<D>& P, const char* k_dq, const char* k_s, const char* v_s,
                                             const char* k_self, const NatOff<D>& no, const TrOff<D>& to,
                                             const bf16x8 (&qf)[1][D / 16], const bf16x8 (&dof)[1][D / 16],
                                             f32x16 (&dq)[1][D / 32], const f32x16& ndelta16, float c) {
  constexpr int N2 = D / 16, NM = LAST ? N2 : N2 + D / 8, O = 1 - KB;
  static_assert(N2 % kDqAhead == 0 && (D / 8) % kDqAhead == 0, "fragment slots must repeat from body to body");
#pragma unroll
  for (int j = 0; j < NM; ++j) {
    const int slot = j % kDqAhead;
    const bf16x8 a = P.ring[slot];
    if (j < N2) {
      dq[0][j % (D / 32)] = mfma32(a, __builtin_bit_cast(bf16x8, P.dsb[O][j / (D / 32)]), dq[0][j % (D / 32)]);
    } else {
      const int i = j - N2, st = i >> 1;
      if (i & 1) P.dpc[O] = mfma32(a, dof[0][st], st == 0 ? ndelta16 : P.dpc[O]);
      else P.sc[O] = mfma32(a, qf[0][st], st == 0 ? zero16() : P.sc[O]);
    }
    if (j + kDqAhead < NM) {
      P.ring[slot] = dq_pipe_frag<D>(k_dq, O, k_s, v_s, O, no, to, j + kDqAhead);
    } else {
      const int jn = j + kDqAhead - NM;
      P.ring[slot] = frag_tr<D>(k_self, to, KB * 32 + (jn / (D / 32)) * 16, jn % (D / 32));
    }
    // Vector work of the unit, skewed by one matrix instruction: p' = 2^(c s) of a few scores here, their
    // products with dP and the rounding to bf16 behind the next instruction, so that neighbouring vector
    // instructions do not depend on one another (registers <-> keys 8*(i/4) + 4g + i%4 of the block).
    // The empty assembly statements keep each value's computation where it is written: without them the
    // compiler moves it to the first use, which for dS is the next body.
    if (j > 0) {
#pragma unroll
      for (int i = 16 * (j - 1) / (NM - 1); i < 16 * j / (NM - 1); ++i) {
        P.sc[KB][i] *= P.dpc[KB][i];
        if (i & 1) {
          uint32_t w = pack_bf16(P.sc[KB][i - 1], P.sc[KB][i]);
          asm volatile("" : "+v"(w));
          P.dsb[KB][i >> 3][(i & 7) >> 1] = w;
        }
      }
    }
    if (j + 1 < NM) {
#pragma unroll
      for (int i = 16 * j / (NM - 1); i < 16 * (j + 1) / (NM - 1); ++i) {
        float e = exp2_fast(P.sc[KB][i] * c);
        asm volatile("" : "+v"(e));
        P.sc[KB][i] = e;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int D, bool SV>
__global__ __launch_bounds__(256, 2) void dq_pipe_kernel(BwdParams p) {
  constexpr int kTileBytes = kKeysPerTile * D * 2;
  constexpr int N2 = D / 16;
  constexpr float kLseRange = 64.f;  // log2 units
  __shared__ __attribute__((aligned(16))) char lds[3][2][kTileBytes];  // [buffer][K|V]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const KeyTileLds<D> kl(&lds[0][0][0], wave);
  const DeviceTileMap& tm = p.tm;
  const int group = p.Hq / p.Hkv;
  int b = blockIdx.x;
  const int kvh = b % p.Hkv;
  b /= p.Hkv;
  const int hc = b % group;
  const int rt = p.rt_hi - 1 - b / group;  // heaviest row tiles first
  const int h = kvh * group + hc;

  const int r = wave * 32 + ln;  // row of the tile owned by this lane (shared with lane ^ 32)
  int tq;
  const bool row_ok = row_token(tm, rt, r, p.L, tq);

  // The K half of the buffer that the first pipelined body reads its (absent) predecessor from: that body
  // multiplies it by dS = 0, so it only has to be finite.
  {
    uint4* z = reinterpret_cast<uint4*>(lds[2][0]);
    for (int i = tid; i < kTileBytes / 16; i += 256) z[i] = make_uint4(0, 0, 0, 0);
  }

  bf16x8 qf[1][D / 16], dof[1][D / 16];
  float lse2, delta;
  {
    const size_t off = ((size_t)(row_ok ? tq : 0) * p.Hq + h) * D + g * 8;
    float dl = 0.f;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const uint4 z = make_uint4(0, 0, 0, 0);
      qf[0][st] = as_frag(row_ok ? ld16(p.q + off + st * 16) : z);
      dof[0][st] = as_frag(row_ok ? ld16(p.d_o + off + st * 16) : z);
      const bf16x8 of = as_frag(row_ok ? ld16(p.o + off + st * 16) : z);
#pragma unroll
      for (int j = 0; j < 8; ++j) dl = __builtin_fmaf((float)dof[0][st][j], (float)of[j], dl);
    }
    delta = sum_halves(dl);
    lse2 = row_ok ? p.lse[(size_t)h * p.T + tq] * kLog2e : 0.f;
    if (row_ok && g == 0) {  // per-row terms in the form the dK/dV kernel consumes
      p.delta[(size_t)h * p.T + tq] = -delta;
      p.nlse[(size_t)h * p.T + tq] = -lse2 / p.c_log2;
    }
  }

  f32x16 dq[1][D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db) dq[0][db] = zero16();

  const NatOff<D> no = nat_offsets<D>(lane);
  const TrOff<D> to = tr_offsets<D>(lane);
  const int e0 = tm.row_ptr[rt], e1 = tm.row_ptr[rt + 1];
  const int n_lead = tm.row_lead[rt];  // leading full tiles
  auto entry_at = [&](int e) { return e < e1 ? e : e1 - 1; };
  TileEntry t_cur = load_entry(tm.row_entries, e0);
  TileEntry t_n1 = load_entry(tm.row_entries, entry_at(e0 + 1));
  TileEntry t_n2 = load_entry(tm.row_entries, entry_at(e0 + 2));

  // the first two tiles are on their way before anything else
  dma_key_tile<D, 4, SV>(kl.k(0), kl.v(0), p.k, p.v, p.Hkv, kvh, tm, t_cur.tile, p.L, wave, lane, p.v_shared);
  if (e0 + 1 < e1) dma_key_tile<D, 4, SV>(kl.k(1), kl.v(1), p.k, p.v, p.Hkv, kvh, tm, t_n1.tile, p.L, wave, lane, p.v_shared);

  // unnormalised probabilities for the whole workgroup, or normalised ones for the whole workgroup
  const bool in_range = __builtin_fabsf(lse2) <= kLseRange;  // (false for NaN)
  const bool unnormalised = __syncthreads_or(row_ok && !in_range) == 0;
  const float lse_used[1] = {unnormalised ? 0.f : lse2};
  const float delta_used[1] = {delta};
  const float row_factor = (unnormalised ? exp2_fast(-lse2) : 1.f) * p.scale;
  const int n_groups = unnormalised ? n_lead / 3 : 0;  // groups of three pipelined tiles

  dma_publish();  // tiles e0 and e0+1 have landed (and the zero fill above is visible)
  int e = e0;

  if (n_groups > 0) {
    f32x16 ndelta16;
#pragma unroll
    for (int i = 0; i < 16; ++i) ndelta16[i] = -delta;
    const float c = p.c_log2;
    DqPipe<D> P;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int t = 0; t < 2; ++t) P.dsb[a][t] = u32x4{0, 0, 0, 0};
    {  // S and dP of the first unit; nothing to overlap them with
      P.sc[0] = zero16();
      P.dpc[0] = ndelta16;
#pragma unroll
      for (int st = 0; st < D / 16; ++st) {
        P.sc[0] = mfma32(frag_nat<D>(lds[0][0], no, 0, st), qf[0][st], P.sc[0]);
        P.dpc[0] = mfma32(frag_nat<D>(lds[0][1], no, 0, st), dof[0][st], P.dpc[0]);
      }
#pragma unroll
      for (int j = 0; j < kDqAhead; ++j) P.ring[j] = dq_pipe_frag<D>(lds[2][0], 1, lds[0][0], lds[0][1], 1, no, to, j);
    }
    // One key tile in buffer B (a compile-time constant).
    auto tile = [&](auto buf_tag, auto last_tag) {
      constexpr int B = decltype(buf_tag)::value, BP = (B + 2) % 3, BN = (B + 1) % 3;
      constexpr bool LAST = decltype(last_tag)::value;
      const u32x2 ahead = fetch_entry(tm.row_entries, entry_at(e + 3));
      dq_pipe_body<D, 0, false>(P, lds[BP][0], lds[B][0], lds[B][1], lds[B][0], no, to, qf, dof, dq, ndelta16, c);
      // Every wave has left tile e-1 (its last reader was the body above) and has waited for its own copies of
      // tile e+1: after the barrier that buffer may be overwritten and tile e+1 may be read.
      dma_publish();
      if (e + 2 < e1) dma_key_tile<D, 4, SV>(kl.k(BP), kl.v(BP), p.k, p.v, p.Hkv, kvh, tm, t_n2.tile, p.L, wave, lane, p.v_shared);
      dq_pipe_body<D, 1, LAST>(P, lds[B][0], lds[BN][0], lds[BN][1], lds[B][0], no, to, qf, dof, dq, ndelta16, c);
      t_cur = t_n1;
      t_n1 = t_n2;
      t_n2 = take_entry(ahead);
      ++e;
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    using B2 = std::integral_constant<int, 2>;
    for (int gi = 0; gi < n_groups - 1; ++gi) {
      tile(B0{}, std::false_type{});
      tile(B1{}, std::false_type{});
      tile(B2{}, std::false_type{});
    }
    tile(B0{}, std::false_type{});
    tile(B1{}, std::false_type{});
    tile(B2{}, std::true_type{});  // starts no further unit
    // dQ of the last unit (block 1 of the tile in buffer 2)
#pragma unroll
    for (int j = 0; j < N2; ++j) {
      const bf16x8 a = j < kDqAhead ? P.ring[j] : frag_tr<D>(lds[2][0], to, 32 + (j / (D / 32)) * 16, j % (D / 32));
      dq[0][j % (D / 32)] = mfma32(a, __builtin_bit_cast(bf16x8, P.dsb[1][j / (D / 32)]), dq[0][j % (D / 32)]);
    }
    // tiles e and e+1 have been copied (e+1 perhaps not yet published), and a wave may still be reading tile e-1
    dma_publish();
  }

  // The remaining tiles, one barrier each: tile e sits in buffer (e - e0) % 3, tile e+1 is published, the
  // copy of tile e+2 goes to the buffer tile e-1 has left.
  int buf = 0;  // (e - e0) % 3: the pipelined part ends on a multiple of three
  for (; e < e1; ++e) {
    const u32x2 ahead = fetch_entry(tm.row_entries, entry_at(e + 3));
    const int buf2 = buf == 0 ? 2 : buf - 1;
    if (e + 2 < e1) dma_key_tile<D, 4, SV>(kl.k(buf2), kl.v(buf2), p.k, p.v, p.Hkv, kvh, tm, t_n2.tile, p.L, wave, lane, p.v_shared);
    const char* kt_lds = lds[0][0] + buf * (2 * kTileBytes);
    const char* vt_lds = kt_lds + kTileBytes;
    if (t_cur.mask_id < 0) {
      const uint32_t mw[2] = {0xffffffffu, 0xffffffffu};
      dq_tile<D, 1, false>(kt_lds, vt_lds, no, to, qf, dof, dq, lse_used, delta_used, mw, p.c_log2);
    } else {
      const u32x2 w = *reinterpret_cast<const u32x2*>(tm.masks + ((size_t)t_cur.mask_id * kRowsPerTile + r) * 2);
      const uint32_t mw[2] = {w[0] >> (4 * g), w[1] >> (4 * g)};
      // a 32-key block that none of the wave's 32 rows can see contributes exact zeros and is left out
      const bool see0 = wave_sees_block(mw[0]), see1 = wave_sees_block(mw[1]);
      if (see0 && see1) dq_tile<D, 1, true>(kt_lds, vt_lds, no, to, qf, dof, dq, lse_used, delta_used, mw, p.c_log2);
      else if (see0) dq_tile<D, 1, true, 0, 1>(kt_lds, vt_lds, no, to, qf, dof, dq, lse_used, delta_used, mw, p.c_log2);
      else if (see1) dq_tile<D, 1, true, 1, 2>(kt_lds, vt_lds, no, to, qf, dof, dq, lse_used, delta_used, mw, p.c_log2);
    }
    dma_publish();
    t_cur = t_n1;
    t_n1 = t_n2;
    t_n2 = take_entry(ahead);
    buf = buf == 2 ? 0 : buf + 1;
  }

  if (row_ok) {
    if (p.rope_table) {
      // q was the rotated copy: turn dQ back.  The lane holds features db*32 + 8*q4 + 4g + j of its
      // row, so both members of every pair (feature, feature + D/2) are in its own registers.
      const float* rope = p.rope_table + (size_t)token_position(tm, tq, p.L) * D;
#pragma unroll
      for (int db = 0; db < D / 64; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = db * 32 + 8 * q4 + 4 * g;
          const f32x4 cs = *reinterpret_cast<const f32x4*>(rope + d0);
          const f32x4 sn = *reinterpret_cast<const f32x4*>(rope + D / 2 + d0);
          f32x4 lo, hi;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            lo[j] = dq[0][db][4 * q4 + j];
            hi[j] = dq[0][db + D / 64][4 * q4 + j];
          }
          rope_turn4<true>(lo, hi, cs, sn);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            dq[0][db][4 * q4 + j] = lo[j];
            dq[0][db + D / 64][4 * q4 + j] = hi[j];
          }
        }
    }
    __bf16* drow = p.dq + ((size_t)tq * p.Hq + h) * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w;
        w[0] = pack_bf16(dq[0][db][4 * q4 + 0] * row_factor, dq[0][db][4 * q4 + 1] * row_factor);
        w[1] = pack_bf16(dq[0][db][4 * q4 + 2] * row_factor, dq[0][db][4 * q4 + 3] * row_factor);
        *reinterpret_cast<u32x2*>(drow + db * 32 + 8 * q4 + 4 * g) = w;
      }
  }
}

// =====================================================================================
// Backward, part 2: dK, dV, key-tile owned.  A workgroup holds a PAIR of adjacent key tiles
// (128 keys) of one KV head in registers and loops over the row tiles that see the first of
// them (clipped to the segment) for the query heads [h_lo, h_hi) assigned to it; the second
// tile's list is a suffix of the first's, so its waves idle on the few leading row tiles.
// Wave w owns key block w (32 keys) and all 128 rows of each row tile.
//   depth-0 key tiles: one query head per workgroup, result to the per-head partial buffer;
//   chain key tiles:   all heads of the KV group, result straight to dk_acc / dv_acc.
// =====================================================================================
// ---- one row tile (128 rows of one query head) against the wave's 32 keys, as one software pipeline ----
// MODE 0: every element visible; 1: key-major bitmask; 2: every element visible except for lanes whose key
// belongs to another sequence of a packed batch (lane_off = true): those lanes contribute nothing.
//
// On this chip a wave that issues a matrix instruction and then independent vector instructions runs the
// vector work in the shadow of the matrix pipe (about four plain vector instructions per
// v_mfma_f32_32x32x16_bf16 cost nothing), whereas matrix and vector phases that follow one another - in the
// same wave or in two waves of one SIMD - take the sum of their times.  The row tile's four 32-row units
// are therefore staggered: while the vector unit turns the scores of unit u into P and dS, the matrix
// pipe runs dV / dK of unit u-1 and S / dP of unit u+1.  The 8 groups of D/8 matrix instructions are
//   S,dP(0) | S,dP(1) | dV,dK(0) | S,dP(2) | dV,dK(1) | S,dP(3) | dV,dK(2) | dV,dK(3)
// and the vector work of units 0..3 rides on groups 1 | 2,3 | 4,5 | 6.  Every matrix instruction is
// followed by its share of vector instructions and a scheduling fence, so the interleaving written here
// is the one the hardware sees; operand fragments are fetched from LDS kPipeAhead instructions ahead.
struct PipeGroup {
  int kind;   // 0: S and dP of `unit`; 1: dV and dK of `unit`
  int unit;   // 32-row block of the row tile
  int vunit;  // unit whose vector work rides on this group (-1: none)
  int e0, e1; // ... and which of its 16 score registers
};
constexpr PipeGroup kPipeGroups[8] = {{0, 0, -1, 0, 0}, {0, 1, 0, 0, 16}, {1, 0, 1, 0, 8},  {0, 2, 1, 8, 16},
                                      {1, 1, 2, 0, 8},  {0, 3, 2, 8, 16}, {1, 2, 3, 0, 16}, {1, 3, -1, 0, 0}};
constexpr int kPipeAhead = 2;

template <int D>
struct DkdvPipe {
  f32x16 sc[2], dpc[2];        // S and dP accumulators of the units in flight (unit & 1)
  u32x4 pb[2][2], dsb[2][2];   // P and dS of a unit as bf16 B operands, per 16-row step
  bf16x8 ring[kPipeAhead];     // A operands on their way from LDS
};

// A operand of matrix instruction j of a group: S / dP read natural fragments (even j: Q, odd j: dO),
// dV / dK transposed ones (even j: dO^T, odd j: Q^T; j/2 = 16-row step * D/32 + feature block).
template <int D, int KIND>
__device__ __forceinline__ bf16x8 pipe_frag(const char* q_lds, const char* do_lds, const NatOff<D>& no,
                                            const TrOff<D>& to, int r0, int j) {
  if (KIND == 0) return *reinterpret_cast<const bf16x8*>(((j & 1) ? do_lds : q_lds) + no.off[j >> 1] + r0 * (2 * D));
  const int idx = j >> 1, db = idx % (D / 32), tt = idx / (D / 32);
  return frag_tr<D>((j & 1) ? q_lds : do_lds, to, r0 + tt * 16, db);
}

// -lse/scale and -Delta of the unit's rows, straight into the accumulators S and dP start from (C layout).
template <int MODE>
__device__ __forceinline__ void pipe_row_terms(f32x16& s, f32x16& dp, const float* nlse_lds, const float* ndelta_lds,
                                               int r0, int g, bool lane_off) {
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const f32x4 l4 = *reinterpret_cast<const f32x4*>(nlse_lds + r0 + 8 * q4 + 4 * g);
    const f32x4 d4 = *reinterpret_cast<const f32x4*>(ndelta_lds + r0 + 8 * q4 + 4 * g);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      s[4 * q4 + j] = MODE == 2 && lane_off ? -__builtin_inff() : l4[j];
      dp[4 * q4 + j] = d4[j];
    }
  }
}

template <int D, int MODE, int G>
__device__ __forceinline__ void dkdv_pipe_group(DkdvPipe<D>& P, const char* q_lds, const char* do_lds,
                                                const float* nlse_lds, const float* ndelta_lds, const NatOff<D>& no,
                                                const TrOff<D>& to, const bf16x8 (&kf)[D / 16],
                                                const bf16x8 (&vf)[D / 16], f32x16 (&dk)[D / 32], f32x16 (&dv)[D / 32],
                                                int g, float c, bool lane_off, const u32x4& cm) {
  constexpr int NG = D / 8;  // matrix instructions per group
  constexpr PipeGroup gd = kPipeGroups[G];
  constexpr PipeGroup gn = kPipeGroups[G + 1 < 8 ? G + 1 : 7];
  constexpr int u = gd.unit & 1, vu = gd.vunit & 1;
  if (G + 1 < 8 && gn.kind == 0)  // the next group starts S / dP of a unit: fetch its per-row terms now
    pipe_row_terms<MODE>(P.sc[gn.unit & 1], P.dpc[gn.unit & 1], nlse_lds, ndelta_lds, gn.unit * 32, g, lane_off);
#pragma unroll
  for (int j = 0; j < NG; ++j) {
    const int slot = (G * NG + j) % kPipeAhead;  // the instruction kPipeAhead later takes the slot this one frees
    const bf16x8 a = P.ring[slot];
    if (gd.kind == 0) {
      if (j & 1) P.dpc[u] = mfma32(a, vf[j >> 1], P.dpc[u]);
      else P.sc[u] = mfma32(a, kf[j >> 1], P.sc[u]);
    } else {
      const int idx = j >> 1, db = idx % (D / 32), tt = idx / (D / 32);
      if (j & 1) dk[db] = mfma32(a, __builtin_bit_cast(bf16x8, P.dsb[u][tt]), dk[db]);
      else dv[db] = mfma32(a, __builtin_bit_cast(bf16x8, P.pb[u][tt]), dv[db]);
    }
    if (j + kPipeAhead < NG)
      P.ring[slot] = pipe_frag<D, gd.kind>(q_lds, do_lds, no, to, gd.unit * 32, j + kPipeAhead);
    else if (G + 1 < 8)
      P.ring[slot] = pipe_frag<D, gn.kind>(q_lds, do_lds, no, to, gn.unit * 32, j + kPipeAhead - NG);
    if (gd.vunit >= 0) {
      const int n = gd.e1 - gd.e0;
#pragma unroll
      for (int i = gd.e0 + n * j / NG; i < gd.e0 + n * (j + 1) / NG; ++i) {
        float pr = exp2_fast(P.sc[vu][i] * c);
        if (MODE == 1) {  // the lane's key-major mask word of this unit: bit of row 8*(i/4) + 4g + i%4
          const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)(cm[gd.vunit & 3] >> (4 * g)), 8 * (i / 4) + (i % 4), 1);
          pr = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, pr) & keep);
        }
        P.sc[vu][i] = pr;
        P.dpc[vu][i] *= pr;
        if (i & 1) {
          P.pb[vu][i >> 3][(i & 7) >> 1] = pack_bf16(P.sc[vu][i - 1], P.sc[vu][i]);
          P.dsb[vu][i >> 3][(i & 7) >> 1] = pack_bf16(P.dpc[vu][i - 1], P.dpc[vu][i]);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int D, int MODE>
__device__ __forceinline__ void dkdv_rowtile_pipelined(const char* q_lds, const char* do_lds, const float* nlse_lds,
                                                       const float* ndelta_lds, const NatOff<D>& no, const TrOff<D>& to,
                                                       const bf16x8 (&kf)[D / 16], const bf16x8 (&vf)[D / 16],
                                                       f32x16 (&dk)[D / 32], f32x16 (&dv)[D / 32], int g, float c,
                                                       bool lane_off = false, const u32x4 cm = u32x4{0, 0, 0, 0}) {
  DkdvPipe<D> P;
  pipe_row_terms<MODE>(P.sc[0], P.dpc[0], nlse_lds, ndelta_lds, 0, g, lane_off);
#pragma unroll
  for (int j = 0; j < kPipeAhead; ++j) P.ring[j] = pipe_frag<D, 0>(q_lds, do_lds, no, to, 0, j);
#define PEAGLE_PIPE_GROUP(G) \
  dkdv_pipe_group<D, MODE, G>(P, q_lds, do_lds, nlse_lds, ndelta_lds, no, to, kf, vf, dk, dv, g, c, lane_off, cm)
  PEAGLE_PIPE_GROUP(0);
  PEAGLE_PIPE_GROUP(1);
  PEAGLE_PIPE_GROUP(2);
  PEAGLE_PIPE_GROUP(3);
  PEAGLE_PIPE_GROUP(4);
  PEAGLE_PIPE_GROUP(5);
  PEAGLE_PIPE_GROUP(6);
  PEAGLE_PIPE_GROUP(7);
#undef PEAGLE_PIPE_GROUP
}

// LISTED: the map names rows by explicit token lists (sampled / packed maps); their tokens are then
// fetched an iteration before the copy that uses them.  A dense map computes them when it issues
// the copy and carries no token registers.
template <int D, bool LISTED, bool SV>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1) void dkdv_kernel(BwdParams p) {
  constexpr int kTileBytes = kRowsPerTile * D * 2;
  constexpr int kBufBytes = 2 * kTileBytes + 2 * kRowsPerTile * 4;  // Q | dO | lse2 | delta
  constexpr int kLdsBytes = 2 * kBufBytes;
  __shared__ __attribute__((aligned(16))) char lds[kLdsBytes];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const int kblk = wave;  // 32-key block of the pair owned by this wave
  const DeviceTileMap& tm = p.tm;
  const int group = p.Hq / p.Hkv;

  int b = blockIdx.x;
  int kt0, n_tiles, kvh, h_lo, h_hi;  // first key tile of the pair, tiles present (1 or 2)
  const bool chain = b >= p.n_d0_items;
  if (!chain) {
    // Workgroups are dealt round-robin to the XCDs, so b % Hkv pins a KV head to an XCD's L2;
    // within it the key-tile pairs of one query head are adjacent, so the workgroups that are
    // resident together stream the same head's Q / dO rows and share them in L2.
    // The pairs are dealt in passes over the heads: pass 0 takes the pairs [0, d0_split), each later
    // pass the next d0_step pairs.  The key tiles inside a segment have lists that shrink with the
    // pair index, and starting the long lists of every head before the short ones lets the short
    // ones fill the slots that free up (one pass - d0_split = pair count - when all lists are
    // equally long).
    const int n_pairs = (p.n_d0_tiles - p.d0_tile_lo + 1) / 2;
    kvh = b % p.Hkv;
    b /= p.Hkv;
    int first = 0, count = p.d0_split;
    while (b >= count * group) {  // at most a few passes
      b -= count * group;
      first += count;
      count = n_pairs - first < p.d0_step ? n_pairs - first : p.d0_step;
    }
    const int pair = first + b % count;
    const int head = b / count;
    kt0 = p.d0_tile_lo + 2 * pair;
    h_lo = kvh * group + head;
    h_hi = h_lo + 1;
    n_tiles = kt0 + 1 < p.n_d0_tiles ? 2 : 1;
  } else {
    b -= p.n_d0_items;
    kvh = b % p.Hkv;
    b /= p.Hkv;
    const int n_cpair = (tm.n_csub + 1) / 2;
    const int sub0 = 2 * (b % n_cpair);
    kt0 = tm.n_d0 + (p.rt_lo + b / n_cpair) * tm.n_csub + sub0;
    n_tiles = sub0 + 1 < tm.n_csub ? 2 : 1;
    h_lo = kvh * group;
    h_hi = h_lo + group;
  }
  const int my_tile = kblk >> 1;             // which tile of the pair this wave's keys belong to
  const int kt = kt0 + my_tile;
  const bool tile_present = my_tile < n_tiles;

  // row tiles that see a key tile, clipped to [rt_lo, rt_hi): the map stores where each segment
  // starts inside a key tile's (ascending) list.  A launch that covers only part of its segments
  // (a cropped length, or one chunk of a long segment; dense maps only) cuts the range further by
  // position: the row tiles in a dense map's list are consecutive.
  auto clip = [&](int t, int& lo_out, int& hi_out) {
    const int32_t* sp = tm.key_seg_ptr + (size_t)t * (tm.S + 1);
    int lo = sp[p.s_lo], hi = sp[p.s_hi];
    if (p.clip_rows && lo < hi) {
      const int first = tm.key_entries[lo].tile;
      const int nlo = lo + (p.rt_lo > first ? p.rt_lo - first : 0);
      const int nhi = lo + (p.rt_hi > first ? p.rt_hi - first : 0);
      lo = nlo < hi ? nlo : hi;
      hi = nhi < hi ? nhi : hi;
    }
    lo_out = lo;
    hi_out = hi;
  };
  int e_lo, e_hi;            // list of the pair's first tile: drives the loop
  clip(kt0, e_lo, e_hi);
  int my_lo = e_lo, my_hi = e_hi;
  if (my_tile == 1 && tile_present) clip(kt, my_lo, my_hi);
  const int n_row_tiles = e_hi - e_lo;
  const int my_skip = tile_present ? n_row_tiles - (my_hi - my_lo) : n_row_tiles;  // leading row tiles that do not see my tile
  const int n_iter = n_row_tiles * (h_hi - h_lo);

  // stationary K, V of this wave's 32 keys: B operands (lane <-> key, registers <-> d)
  bf16x8 kf[D / 16], vf[D / 16];
  int key_tok = 0;
  const bool key_ok = tile_present && key_token(tm, kt, (kblk & 1) * 32 + ln, p.L, key_tok);
  const int key_anchor = kt * kKeysPerTile + (kblk & 1) * 32 + ln;  // meaningful for depth-0 tiles only
  {
    const size_t off = ((size_t)(key_ok ? key_tok : 0) * p.Hkv + kvh) * D + g * 8;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) {
      const uint4 z = make_uint4(0, 0, 0, 0);
      const __bf16* vrow = SV && chain ? p.v_shared + (size_t)kvh * D + g * 8 : p.v + off;
      const uint4 a = ld16(p.k + off + st * 16), c = ld16(vrow + st * 16);
      kf[st] = as_frag(key_ok ? a : z);
      vf[st] = as_frag(key_ok ? c : z);
    }
  }

  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    dk[db] = zero16();
    dv[db] = zero16();
  }

  const NatOff<D> no = nat_offsets<D>(lane);
  const TrOff<D> to = tr_offsets<D>(lane);

  // Q / dO row tiles and their per-row terms (-lse/scale, -Delta, prepared by the dQ kernel) go
  // straight from global memory into the LDS buffer that the next iteration reads.
  const RowDmaLane<D, 4> rl = row_dma_lane<D, 4>(tm, p.L, wave, lane, p.Hq);
  using Toks = RowTokens<D, 4>;
  // dense map whose row tiles hold 128 real rows, tensors within reach of a 32-bit offset: copies of whole row
  // tiles take the short form
  const bool fast_rows = !LISTED && tm.A * tm.K == kRowsPerTile && p.fast_rows;
  // The rows a lane copies are kRowsApart apart; when that is a whole number of depths (A divides it), copy i
  // reads fast_step elements behind copy i-1 for every lane: the step goes into the scalar base and one per-lane
  // offset serves all copies.  Otherwise (fast_step = 0) each copy has its own per-lane offset.
  constexpr int kRowsApart = 4 * (512 / D);
  const size_t fast_step = kRowsApart % tm.A == 0 ? (size_t)(kRowsApart / tm.A) * p.L * p.Hq * D : 0;
  // Everything but the one per-lane offset is computed on the scalar unit from values forced wave-uniform (the
  // compiler otherwise carries the row tile and head in vector registers and builds each copy's 64-bit
  // address there): LDS addresses are plain integers from the buffer's base, the source pointers scalar
  // multiplies and adds, and the choice between the two forms is made once, not per copy.
  const uint32_t lds_addr0 = lds_scalar_addr(lds);
  const uint32_t wave_s = (uint32_t)__builtin_amdgcn_readfirstlane(wave);
  constexpr int kPer = RowDmaLane<D, 4>::kPer;
  auto issue_fast = [&](int hh, int rt, int buf) {
    const int hh_s = __builtin_amdgcn_readfirstlane(hh), rt_s = __builtin_amdgcn_readfirstlane(rt);
    const uint32_t dst = lds_addr0 + (uint32_t)buf * kBufBytes + wave_s * 1024;
    const size_t row0 = ((size_t)rt_s * tm.A * p.Hq + hh_s) * D;
    const __bf16* qs = p.q + row0;
    const __bf16* ds = p.d_o + row0;
    if (fast_step) {
#pragma unroll
      for (int i = 0; i < kPer; ++i) dma16_untracked(qs + i * fast_step, rl.fast_off[0], dst + i * 4 * 1024);
#pragma unroll
      for (int i = 0; i < kPer; ++i) dma16_untracked(ds + i * fast_step, rl.fast_off[0], dst + kTileBytes + i * 4 * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < kPer; ++i) dma16_untracked(qs, rl.fast_off[i], dst + i * 4 * 1024);
#pragma unroll
      for (int i = 0; i < kPer; ++i) dma16_untracked(ds, rl.fast_off[i], dst + kTileBytes + i * 4 * 1024);
    }
    const float* stat0 = (wave_s < 2 ? p.nlse : p.delta) + (size_t)hh_s * p.T + (size_t)rt_s * tm.A;
    dma4_untracked(stat0, rl.fast_stat_off,
                   lds_addr0 + (uint32_t)buf * kBufBytes + 2 * kTileBytes + (wave_s < 2 ? 0 : kRowsPerTile * 4) +
                       (wave_s & 1) * 64 * 4);
  };
  auto issue = [&](int hh, const Toks& t, int buf) {
    char* base = lds + buf * kBufBytes;
    dma_row_tile<D, 4>(base, p.q, p.Hq, hh, tm, rl, t, wave);
    dma_row_tile<D, 4>(base + kTileBytes, p.d_o, p.Hq, hh, tm, rl, t, wave);
    float* stat = reinterpret_cast<float*>(base + 2 * kTileBytes);
    if (wave < 2) dma_row_stat<D, 4>(stat, p.nlse, p.T, hh, tm, t, wave & 1);
    else if (wave < 4) dma_row_stat<D, 4>(stat + kRowsPerTile, p.delta, p.T, hh, tm, t, wave & 1);
  };
  // Iteration `it` handles row tile ei = it % n_row_tiles of head h_lo + it / n_row_tiles.  The
  // pipeline runs three deep: the list entry of iteration it+3 is fetched now and moved to scalar
  // registers after the barrier; the row tokens of it+2 are fetched now (they need that
  // iteration's row tile); the copy of it+1 is issued now; the mask of it+2 is fetched now.  Key-
  // side mask ids: -1 every element visible, >= 0 a bitmask, INT_MIN nothing to do (a row tile
  // that does not see this wave's key tile; also set by the map for row tiles listed only for the
  // other tile of the pair), other ids <= -2 visible for keys with anchor >= -id - 2 (the row
  // tile's sequence starts inside the key tile).
  // The list is walked from its last row tile down: every key tile of a launch ends at the same
  // row tile, so workgroups of one head that start together then read the same Q / dO rows at the
  // same time (they share them in L2) whether their lists are long or short.
  auto list_pos = [&](int ei) { return n_row_tiles - 1 - ei; };
  auto fetch_row_tile = [&](int ei) { return fetch_entry(tm.key_entries, e_lo + list_pos(ei)); };
  auto fetch_mask = [&](int ei) {
    const int li = list_pos(ei);
    return fetch_entry(tm.key_entries, li >= my_skip ? my_lo + li - my_skip : e_lo + li);
  };
  constexpr int kSkip = INT_MIN;
  auto mask_of = [&](int ei, const TileEntry& en) {  // (wave-uniform: through readfirstlane so that it stays scalar)
    return list_pos(ei) >= my_skip ? en.mask_id : kSkip;
  };
  auto step = [&](int& ei, int& hh) {  // advance (ei, hh) by one iteration
    if (++ei == n_row_tiles) {
      ei = 0;
      ++hh;
    }
  };

  int ei_n = 0, hh_n = h_lo;        // iteration it+1 (its copy is issued now)
  int ei_a = 0, hh_a = h_lo;        // it+2 (its row tokens and mask are fetched now)
  int ei_b = 0, hh_b = h_lo;        // it+3 (its list entry is fetched now)
  int rt_n = 0, rt_a = 0, mask_c = kSkip, mask_n = kSkip;
  Toks tok_n{};
  if (n_iter > 0) {
    const Toks t0 = row_tokens<D, 4, LISTED>(tm, rl, take_entry(fetch_row_tile(0)).tile, p.L);
    issue(h_lo, t0, 0);
    tok_n = t0;
    mask_c = mask_of(0, take_entry(fetch_mask(0)));
    step(ei_n, hh_n);
    step(ei_a, hh_a);
    step(ei_a, hh_a);
    step(ei_b, hh_b);
    step(ei_b, hh_b);
    step(ei_b, hh_b);
    if (n_iter > 1) {
      rt_n = take_entry(fetch_row_tile(ei_n)).tile;
      if (LISTED) tok_n = row_tokens<D, 4, LISTED>(tm, rl, rt_n, p.L);
      mask_n = mask_of(ei_n, take_entry(fetch_mask(ei_n)));
    }
    if (n_iter > 2) rt_a = take_entry(fetch_row_tile(ei_a)).tile;
  }
  dma_publish();

  for (int it = 0; it < n_iter; ++it) {
    const int buf = it & 1;
    const bool have2 = it + 2 < n_iter, have3 = it + 3 < n_iter;
    Toks tok_a = tok_n;
    if (LISTED) {
      if (have2) tok_a = row_tokens<D, 4, LISTED>(tm, rl, rt_a, p.L);
      if (it + 1 < n_iter) issue(hh_n, tok_n, buf ^ 1);
    } else {
      if (it + 1 < n_iter) {
        if (fast_rows && (rt_n + 1) * tm.A <= p.L) issue_fast(hh_n, rt_n, buf ^ 1);
        else issue(hh_n, row_tokens<D, 4, LISTED>(tm, rl, rt_n, p.L), buf ^ 1);
      }
    }
    // (fetched after the copies were issued: anything the copy code has to wait for - a reloaded register -
    // then finds no list load in flight)
    const u32x2 rt_raw = fetch_row_tile(have3 ? ei_b : 0);
    const u32x2 mask_raw = fetch_mask(have2 ? ei_a : 0);
    if (mask_c != kSkip) {
      const char* q_lds = lds + buf * kBufBytes;
      const char* do_lds = q_lds + kTileBytes;
      const float* lse_lds = reinterpret_cast<const float*>(q_lds + 2 * kTileBytes);
      const float* delta_lds = lse_lds + kRowsPerTile;
      if (mask_c == -1) {
        dkdv_rowtile_pipelined<D, 0>(q_lds, do_lds, lse_lds, delta_lds, no, to, kf, vf, dk, dv, g, p.c_log2);
      } else if (mask_c >= 0) {
        // which of the tile's 128 rows see this lane's key: four words, one per 32-row unit
        // (scalar base + small per-lane offset: no 64-bit per-lane address is kept across the loop)
        const uint32_t* mbase = uniform_ptr(tm.masks_by_key + (size_t)__builtin_amdgcn_readfirstlane(mask_c) * kMaskWords);
        const u32x4 cm = *reinterpret_cast<const u32x4*>(mbase + ((kblk & 1) * 32 + ln) * 4);
        dkdv_rowtile_pipelined<D, 1>(q_lds, do_lds, lse_lds, delta_lds, no, to, kf, vf, dk, dv, g, p.c_log2, false, cm);
      } else if (LISTED) {  // only packed maps carry such ids
        const bool lane_off = key_anchor < -mask_c - 2;
        dkdv_rowtile_pipelined<D, 2>(q_lds, do_lds, lse_lds, delta_lds, no, to, kf, vf, dk, dv, g, p.c_log2, lane_off);
      }
    }
    dma_publish();
    if (LISTED) tok_n = tok_a;
    rt_n = rt_a;
    rt_a = take_entry(rt_raw).tile;
    mask_c = mask_n;
    mask_n = have2 ? mask_of(ei_a, take_entry(mask_raw)) : kSkip;
    step(ei_n, hh_n);
    step(ei_a, hh_a);
    step(ei_b, hh_b);
  }

  if (SV && chain) {
    // First-layer form: the chain keys' gradients are only ever needed summed over the keys (they all come from
    // one shared vector), so each wave adds up its 32 keys here - dK after it has been turned back to the
    // unrotated frame, key by key - and stores one row of D sums per tensor.  The sum over keys runs across
    // lanes: the wave lays its values out in LDS as [d][key] (33 floats per d: conflict-free both ways) and lane
    // l adds up row d = l (and l + 64).  The row tiles' buffers are free: every wave is past the loop's last
    // barrier.  Keys that do not exist contribute zero.
    float* red = reinterpret_cast<float*>(lds) + (size_t)wave * (D * 33);
    static_assert(4 * D * 33 * 4 <= kLdsBytes, "the four waves' transposition buffers must fit");
    const bool have = tile_present && key_ok;
    const float* rope = p.rope_table && have ? p.rope_table + (size_t)token_position(tm, key_tok, p.L) * D : nullptr;
    const int b_chain = (int)blockIdx.x - p.n_d0_items;
    const int n_cpair = (tm.n_csub + 1) / 2;
    const size_t prow = ((size_t)(p.rt_lo + b_chain / p.Hkv / n_cpair) * n_cpair + (b_chain / p.Hkv) % n_cpair) * 4 + wave;
#pragma unroll
    for (int which = 0; which < 2; ++which) {  // 0: dK, 1: dV
      if (which == 0 && rope) {
#pragma unroll
        for (int db = 0; db < D / 64; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int d0 = db * 32 + 8 * q4 + 4 * g;
            f32x4 lo, hi;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              lo[j] = dk[db][4 * q4 + j];
              hi[j] = dk[db + D / 64][4 * q4 + j];
            }
            rope_turn4<true>(lo, hi, *reinterpret_cast<const f32x4*>(rope + d0),
                             *reinterpret_cast<const f32x4*>(rope + D / 2 + d0));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              dk[db][4 * q4 + j] = lo[j];
              dk[db + D / 64][4 * q4 + j] = hi[j];
            }
          }
      }
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int d = db * 32 + 8 * (i / 4) + 4 * g + (i % 4);
          const float x = which ? dv[db][i] : dk[db][i] * p.scale;
          red[d * 33 + ln] = have ? x : 0.f;
        }
      asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");  // the wave's own LDS writes have landed
      float* out = (which ? p.shared_dv_part : p.shared_dk_part) + (prow * p.Hkv + kvh) * D;
#pragma unroll
      for (int d = lane; d < D; d += 64) {
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) sum += red[d * 33 + j];
        out[d] = sum;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");  // ... and its reads, before the buffer is written again
    }
    return;
  }

  // store from registers: lane <-> key, registers <-> d = db*32 + 8*q4 + 4g + j
  if (tile_present) {
    float* dkd;
    float* dvd;
    bool write = true, accumulate = false;
    if (!chain) {
      const size_t row = (size_t)h_lo * p.L64 + (size_t)kt * kKeysPerTile + (kblk & 1) * 32 + ln;
      dkd = p.dk_part + row * D;
      dvd = p.dv_part + row * D;
    } else {
      write = key_ok;
      accumulate = p.chain_accumulate != 0;
      const size_t row = (size_t)(key_ok ? key_tok : 0) * p.Hkv + kvh;
      dkd = p.dk_acc + row * D;
      dvd = p.dv_acc + row * D;
    }
    if (write && chain && p.rope_table) {
      // k was the rotated copy: turn the chain keys' dK back (lane <-> key, both members of a feature
      // pair in its registers).  Depth-0 keys are turned back where their per-head partials are summed.
      const float* rope = p.rope_table + (size_t)token_position(tm, key_tok, p.L) * D;
#pragma unroll
      for (int db = 0; db < D / 64; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = db * 32 + 8 * q4 + 4 * g;
          f32x4 lo, hi;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            lo[j] = dk[db][4 * q4 + j];
            hi[j] = dk[db + D / 64][4 * q4 + j];
          }
          rope_turn4<true>(lo, hi, *reinterpret_cast<const f32x4*>(rope + d0),
                           *reinterpret_cast<const f32x4*>(rope + D / 2 + d0));
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            dk[db][4 * q4 + j] = lo[j];
            dk[db + D / 64][4 * q4 + j] = hi[j];
          }
        }
    }
    if (write) {
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 a, c;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            a[j] = dk[db][4 * q4 + j] * p.scale;
            c[j] = dv[db][4 * q4 + j];
          }
          const int d0 = db * 32 + 8 * q4 + 4 * g;
          if (accumulate) {
            a += *reinterpret_cast<const f32x4*>(dkd + d0);
            c += *reinterpret_cast<const f32x4*>(dvd + d0);
          }
          *reinterpret_cast<f32x4*>(dkd + d0) = a;
          *reinterpret_cast<f32x4*>(dvd + d0) = c;
        }
    }
  }
}

// Sum the per-head partials of the depth-0 keys [key_first, key_end) over each KV group into
// dk_acc / dv_acc; keys with anchor < acc_below are added to, the others overwritten.
template <int D>
__global__ __launch_bounds__(256) void reduce_partials_kernel(BwdParams p, int key_first, int key_end, int acc_below) {
  const int group = p.Hq / p.Hkv;
  const size_t per = (size_t)(key_end - key_first) * p.Hkv * (D / 4);
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < 2 * per; idx += (size_t)gridDim.x * blockDim.x) {
    const int which = idx >= per;
    size_t rem = which ? idx - per : idx;
    const int c4 = rem % (D / 4);
    rem /= (D / 4);
    const int kvh = rem % p.Hkv;
    const int j = key_first + (int)(rem / p.Hkv);
    const float* part = which ? p.dv_part : p.dk_part;
    // With rotary embedding the summed dK is turned back to the unrotated keys' frame: the thread of
    // a lower-half piece also sums its partner piece of the upper half and stores both.
    const bool turn = !which && p.rope_table != nullptr;
    if (turn && c4 >= D / 8) continue;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f}, sum_hi = {0.f, 0.f, 0.f, 0.f};
    for (int hh = 0; hh < group; ++hh) {
      const float* src = part + (((size_t)(kvh * group + hh) * p.L64 + j) * D + c4 * 4);
      sum += *reinterpret_cast<const f32x4*>(src);
      if (turn) sum_hi += *reinterpret_cast<const f32x4*>(src + D / 2);
    }
    float* dst = (which ? p.dv_acc : p.dk_acc) + (((size_t)j * p.Hkv + kvh) * D + c4 * 4);
    if (turn) {
      const float* rope = p.rope_table + (size_t)token_position(p.tm, j, p.L) * D + c4 * 4;  // depth-0 key j is token j
      rope_turn4<true>(sum, sum_hi, *reinterpret_cast<const f32x4*>(rope), *reinterpret_cast<const f32x4*>(rope + D / 2));
      if (j < acc_below) sum_hi += *reinterpret_cast<const f32x4*>(dst + D / 2);
      *reinterpret_cast<f32x4*>(dst + D / 2) = sum_hi;
    }
    if (j < acc_below) sum += *reinterpret_cast<const f32x4*>(dst);
    *reinterpret_cast<f32x4*>(dst) = sum;
  }
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* src, __bf16* dst, size_t n4) {
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n4; idx += (size_t)gridDim.x * blockDim.x) {
    const f32x4 x = *reinterpret_cast<const f32x4*>(src + idx * 4);
    u32x2 w;
    w[0] = pack_bf16(x[0], x[1]);
    w[1] = pack_bf16(x[2], x[3]);
    *reinterpret_cast<u32x2*>(dst + idx * 4) = w;
  }
}

// =====================================================================================
// Inference-side drafting step: the K new rows of a request (depth 0 = next-token position, depths
// 1..K-1 = multi-token positions, all of the anchor that follows the cached context) are the last
// anchor's rows of the parallel-prediction mask: every cached key is visible, and the new key of
// depth e is visible to the rows of depth >= e.  One workgroup per (context split, KV head,
// request); its waves own 32 rows each of the K x (Hq/Hkv) query rows that share the KV head
// (row = depth * group + head), loop over the split's 64-token pages with the forward's tile
// routine, and leave an unnormalised partial (reference max, row sum, O) for the combine kernel.
// The work is bound by reading the cache once; the matrix cores only keep the arithmetic off
// the critical path.
// =====================================================================================
template <int D, int kRing>
__global__ __launch_bounds__(320) void draft_decode_kernel(DecodeParams p) {
  constexpr int kTileBytes = kKeysPerTile * D * 2;
  constexpr int kBlocks = kTileBytes / 1024;
  // kRing LDS buffers of one tile (K and V) each: two, or four at D = 64 when a workgroup has many tiles
  constexpr int kCopiesPerTile = 2 * kBlocks;
  static_assert((kRing - 2) * kCopiesPerTile <= 63, "the copies in flight behind a tile must fit the hardware's counter");
  __shared__ __attribute__((aligned(16))) char lds[kRing][2][kTileBytes];  // [buffer][K|V]
  __shared__ int tile_keys[kRing];  // keys present in the tile of each buffer (0 .. 64), set by the copying wave
  __shared__ int table_bad;         // the copying wave met a page id outside the pool

  // The last wave of the workgroup only copies (global -> LDS), the others only compute.  The wait for
  // a copy is counted per wave and in issue order, so the copying wave keeps kRing - 1 tiles in flight
  // and waits for the oldest alone, and the computing waves never wait on a copy.  One workgroup barrier
  // per tile hands the buffers over.
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const int n_compute = (blockDim.x >> 6) - 1;
  const bool producer = wave == n_compute;
  const int split = blockIdx.x, kvh = blockIdx.y, c = blockIdx.z;
  const int group = p.Hq / p.Hkv;
  const int n_rows = p.K * group;

  // context of this request, clamped to what the block table can describe
  int n_ctx = p.ctx_len[c];
  bool bad = n_ctx < 0 || n_ctx > p.max_pages * kKeysPerTile;
  n_ctx = n_ctx < 0 ? 0 : (n_ctx > p.max_pages * kKeysPerTile ? p.max_pages * kKeysPerTile : n_ctx);
  const int n_pg = (n_ctx + kKeysPerTile - 1) / kKeysPerTile;
  const int per = (n_pg + p.n_splits - 1) / p.n_splits;
  const int p0 = split * per < n_pg ? split * per : n_pg;
  const int p1 = p0 + per < n_pg ? p0 + per : n_pg;
  const int n_tiles = (p1 - p0) + (split == 0 ? 1 : 0);  // split 0 also takes the new keys

  // Tile i of this split is a cache page or, last in split 0, the K new keys.  Only the copying wave
  // reads the block table - through the scalar (constant) path, because a vector load would be ordered
  // behind its copies and using the result would wait for all of them, and one tile ahead of its use,
  // so that the load's latency is off the path; it tells the computing waves how many keys each tile
  // holds through tile_keys[] (a page id outside the pool makes the tile empty and flags the request).
  typedef const int32_t __attribute__((address_space(4))) * ConstTable;
  auto page_of = [&](int i) {
    return i < p1 - p0 ? ((ConstTable)(uintptr_t)p.block_table)[(size_t)c * p.max_pages + p0 + i] : 0;
  };

  if (producer) {
    // Rows of a tile that hold no key (tail of the last page, rows past the K new keys, an empty tile)
    // are filled from the request's first new key, which is always present and finite user data: their
    // probabilities are masked to zero, and zero times a finite value adds nothing.
    const __bf16* k_fill = p.k_new + ((size_t)c * p.K * p.Hkv + kvh) * D;
    const __bf16* v_fill = p.v_new + ((size_t)c * p.K * p.Hkv + kvh) * D;
    const int row_in_blk = lane / (D / 8), phys = lane % (D / 8);
    int page_next = page_of(0);
    auto copy_tile = [&](int i) {
      const int page = page_next;
      page_next = page_of(i + 1);
      const bool is_new = i >= p1 - p0;
      int valid = p.K;
      if (!is_new) {
        valid = n_ctx - (p0 + i) * kKeysPerTile;
        valid = valid > kKeysPerTile ? kKeysPerTile : valid;
        if (page < 0 || page >= p.n_pages) {
          bad = true;
          valid = 0;
        }
      }
      if (lane == 0) tile_keys[i % kRing] = valid;
      // (untracked copies: a tracked one would make every workgroup barrier below wait for all of them)
      const uint32_t kdst = lds_scalar_addr(lds[i % kRing][0]), vdst = lds_scalar_addr(lds[i % kRing][1]);
#pragma unroll 4
      for (int blk = 0; blk < kBlocks; ++blk) {
        const int row = blk * (512 / D) + row_in_blk;
        const int chunk = (phys ^ swz<D>(row)) << 3;
        const __bf16 *ks, *vs;
        if (row >= valid) {
          ks = k_fill + chunk;
          vs = v_fill + chunk;
        } else if (is_new) {
          ks = k_fill + (size_t)row * p.Hkv * D + chunk;
          vs = v_fill + (size_t)row * p.Hkv * D + chunk;
        } else {
          const size_t off = (((size_t)page * p.Hkv + kvh) * kKeysPerTile + row) * D + chunk;
          ks = p.k_pages + off;
          vs = p.v_pages + off;
        }
        dma16_untracked(ks, kdst + blk * 1024);
        dma16_untracked(vs, vdst + blk * 1024);
      }
    };
    int issued = 0;
    for (; issued < n_tiles && issued < kRing - 1; ++issued) copy_tile(issued);
    for (int i = 0; i < n_tiles; ++i) {
      // Tile i must have landed; the `later` tiles issued behind it may still be in flight.  Copies
      // complete in issue order, so waiting until at most later * kCopiesPerTile accesses are outstanding
      // is enough (anything else this wave may have in flight only makes the wait longer).
      const int later = issued - 1 - i;  // 0 .. kRing - 2
      if (later >= 2) wait_outstanding<kRing >= 4 ? 2 * kCopiesPerTile : 0>();
      else if (later == 1) wait_outstanding<kCopiesPerTile>();
      else wait_outstanding<0>();
      if (i == n_tiles - 1 && lane == 0) table_bad = bad ? 1 : 0;  // every tile has been looked up by now
      __syncthreads();  // tile i is published; the computing waves are done with tile i-1 ...
      if (issued < n_tiles) copy_tile(issued++);  // ... whose buffer takes tile i + kRing - 1
    }
    if (n_tiles == 0) {
      if (lane == 0) table_bad = 0;
      __syncthreads();
    }
    return;  // barriers executed: max(n_tiles, 1), the same as the computing waves below
  }

  const int r = wave * 32 + ln;  // query row of this lane (shared with lane ^ 32)
  const bool row_ok = r < n_rows;
  const int depth = row_ok ? r / group : 0, head = kvh * group + (row_ok ? r - depth * group : 0);
  bf16x8 qf[1][D / 16];
  {
    const __bf16* qrow = p.q_new + (((size_t)c * p.K + depth) * p.Hq + head) * D + g * 8;
#pragma unroll
    for (int st = 0; st < D / 16; ++st) qf[0][st] = as_frag(ld16(qrow + st * 16));
  }
  f32x16 o[1][D / 32];
  float m[1] = {kNegInit}, lsum[1] = {0.f};
#pragma unroll
  for (int db = 0; db < D / 32; ++db) o[0][db] = zero16();
  const NatOff<D> no = nat_offsets<D>(lane);
  const TrOff<D> to = tr_offsets<D>(lane);

  if (n_tiles == 0) __syncthreads();
  for (int i = 0; i < n_tiles; ++i) {
    __syncthreads();  // tile i has landed
    const int buf = i % kRing;
    const bool is_new = i >= p1 - p0;
    const int valid = __builtin_amdgcn_readfirstlane(tile_keys[buf]);
    if (!is_new && valid == kKeysPerTile) {
      const uint32_t mw[2] = {0xffffffffu, 0xffffffffu};
      fwd_tile<D, 1, false, true>(lds[buf][0], lds[buf][1], no, to, qf, o, m, lsum, mw, p.c_log2);
    } else {
      // keys [0, n) of the tile are visible: n = the page's valid tokens, or depth + 1 of the new keys
      const int n = is_new ? depth + 1 : valid;
      const uint64_t bits = n >= 64 ? ~0ull : ((1ull << n) - 1);
      const uint32_t mw[2] = {(uint32_t)bits >> (4 * g), (uint32_t)(bits >> 32) >> (4 * g)};
      fwd_tile<D, 1, true, true>(lds[buf][0], lds[buf][1], no, to, qf, o, m, lsum, mw, p.c_log2);
    }
  }

  // partial record of this split: lane <-> row, registers <-> d = db*32 + 8*q4 + 4g + j
  const float l_tot = sum_halves(lsum[0]);
  const size_t rec = ((size_t)c * p.Hkv + kvh) * p.n_splits + split;
  if (r < p.rows_pad) {
    float* po = p.part_o + (rec * p.rows_pad + r) * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 a;
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] = o[0][db][4 * q4 + j];
        *reinterpret_cast<f32x4*>(po + db * 32 + 8 * q4 + 4 * g) = a;
      }
    if (g == 0) {
      float* ml = p.part_ml + rec * 3 * p.rows_pad;
      ml[r] = m[0];
      ml[p.rows_pad + r] = l_tot;
      ml[2 * p.rows_pad + r] = (bad || table_bad != 0) ? 1.f : 0.f;  // (table_bad: written before the last barrier)
    }
  }
}

// Merges the splits of a request's rows: M = max m_s, L = sum l_s 2^(m_s - M), O = sum O_s 2^(m_s - M) / L.
// One thread per (request, KV head, row, 4 features).  The loads of a batch of splits are issued
// together (the loops are unrolled in batches with clamped indices): a thread's time is a few memory
// round trips, not one per split.  Block 0 also sets the per-request status words, a wave per request.
template <int D>
__global__ __launch_bounds__(256) void draft_decode_combine_kernel(DecodeParams p) {
  constexpr int kBatch = 8;
  const int group = p.Hq / p.Hkv;
  const int n_rows = p.K * group;
  const size_t n = (size_t)p.C * p.Hkv * n_rows * (D / 4);
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
    const int c4 = (int)(idx % (D / 4));
    size_t rem = idx / (D / 4);
    const int r = (int)(rem % n_rows);
    rem /= n_rows;
    const int kvh = (int)(rem % p.Hkv);
    const int c = (int)(rem / p.Hkv);
    const size_t rec0 = ((size_t)c * p.Hkv + kvh) * p.n_splits;
    const float* ml0 = p.part_ml + rec0 * 3 * p.rows_pad + r;
    const float* o0 = p.part_o + (rec0 * p.rows_pad + r) * D + c4 * 4;
    float M = kNegInit;
    for (int s0 = 0; s0 < p.n_splits; s0 += kBatch) {
      float mv[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int s = s0 + j < p.n_splits ? s0 + j : p.n_splits - 1;
        mv[j] = ml0[(size_t)s * 3 * p.rows_pad];
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) M = __builtin_fmaxf(M, mv[j]);
    }
    float L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < p.n_splits; s0 += kBatch) {
      float mv[kBatch], lv[kBatch];
      f32x4 ov[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int s = s0 + j < p.n_splits ? s0 + j : p.n_splits - 1;
        mv[j] = ml0[(size_t)s * 3 * p.rows_pad];
        lv[j] = ml0[(size_t)s * 3 * p.rows_pad + p.rows_pad];
        ov[j] = *reinterpret_cast<const f32x4*>(o0 + (size_t)s * p.rows_pad * D);
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const float w = s0 + j < p.n_splits ? exp2_fast(mv[j] - M) : 0.f;
        L = __builtin_fmaf(lv[j], w, L);
        acc += ov[j] * w;
      }
    }
    const float inv = 1.0f / L;
    const int depth = r / group, head = kvh * group + (r - depth * group);
    u32x2 w2;
    w2[0] = pack_bf16(acc[0] * inv, acc[1] * inv);
    w2[1] = pack_bf16(acc[2] * inv, acc[3] * inv);
    *reinterpret_cast<u32x2*>(p.o + (((size_t)c * p.K + depth) * p.Hq + head) * D + c4 * 4) = w2;
    if (c4 == 0) p.lse[((size_t)c * p.Hq + head) * p.K + depth] = (M + __builtin_log2f(L)) * kLn2;
  }
  if (p.status && blockIdx.x == 0) {
    // a request is flagged if any of its workgroups met a bad block-table entry or length
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwv = blockDim.x >> 6;
    const int per_req = p.Hkv * p.n_splits;
    for (int c = wave; c < p.C; c += nwv) {
      bool any = false;
      for (int w = lane; w < per_req; w += 64)
        any |= p.part_ml[((size_t)c * per_req + w) * 3 * p.rows_pad + 2 * p.rows_pad] != 0.f;
      const bool flagged = __builtin_amdgcn_ballot_w64(any) != 0;
      if (lane == 0) p.status[c] = flagged ? 1 : 0;
    }
  }
}

// ------------------------------------------------------------------------------------- launchers

// Pure MFMA issue loop (no memory traffic): four independent accumulator chains per wave,
// 8 workgroups x 4 waves per CU.  Used only to report the measured matrix-core ceiling.
// RANDOM = false: small integer operands that never change (little switching activity in the multipliers);
// RANDOM = true: four sets of operands drawn from a hash, roughly uniform in (-2, 2) with every significand
// bit in use, taken in turn - the activity the matrix cores see on real Q, K, V.  The chip lowers its clock
// under the second kind of load, so the two rates differ.
template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(float* out, int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (RANDOM) {
        uint32_t x = (blockIdx.x * 256u + threadIdx.x) * 64u + s * 16u + j;
        x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
        a[s][j] = (__bf16)(((float)(x & 0xffffu) - 32767.5f) * (2.0f / 32768.0f));
        b[s][j] = (__bf16)(((float)(x >> 16) - 32767.5f) * (2.0f / 32768.0f));
      } else {
        a[s][j] = (__bf16)(float)(threadIdx.x % 3);
        b[s][j] = (__bf16)(float)(threadIdx.x % 5);
      }
    }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = zero16();
  for (int it = 0; it < iters; it += 4) {  // (iters is a multiple of four)
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = mfma32(a[RANDOM ? i : 0], b[RANDOM ? (i + u) & 3 : 0], acc[i]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

namespace {

// Query heads of one KV group that share a workgroup's K/V tiles in the forward: two at D = 64 (the register
// budget of two waves per SIMD allows it), one at D = 128.  The backward kernels take one head per workgroup.
inline int pick_nh(int group, int D) { return (D == 64 && group % 2 == 0) ? 2 : 1; }

struct TimedSpan {
  KernelTimer* t;
  hipStream_t stream;
  hipError_t err = hipSuccess;
  TimedSpan(KernelTimer* timer, int kind, hipStream_t s) : t(timer), stream(s) {
    if (t) err = t->begin(kind, s);
  }
  hipError_t finish() {
    hipError_t e = hipGetLastError();
    if (t && err == hipSuccess) err = t->end(stream);
    return e != hipSuccess ? e : err;
  }
};

}  // namespace

hipError_t KernelTimer::begin(int kind, hipStream_t stream) {
  Span sp{nullptr, nullptr, kind};
  hipError_t e = hipEventCreate(&sp.start);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&sp.stop);
  if (e != hipSuccess) {
    (void)hipEventDestroy(sp.start);
    return e;
  }
  spans.push_back(sp);
  return hipEventRecord(sp.start, stream);
}

hipError_t KernelTimer::end(hipStream_t stream) { return hipEventRecord(spans.back().stop, stream); }

hipError_t KernelTimer::collect(float* ms, int32_t* launches) {
  hipError_t rc = hipSuccess;
  for (Span& sp : spans) {
    float t = 0.f;
    hipError_t e = hipEventSynchronize(sp.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, sp.start, sp.stop);
    if (e == hipSuccess) {
      ms[sp.kind] += t;
      launches[sp.kind] += 1;
    } else {
      rc = e;
    }
  }
  return rc;
}

KernelTimer::~KernelTimer() {
  for (Span& sp : spans) {
    (void)hipEventDestroy(sp.start);
    (void)hipEventDestroy(sp.stop);
  }
}

hipError_t launch_fwd(const FwdParams& p, int D, hipStream_t stream, KernelTimer* timer) {
  const int n_rt = p.rt_hi - p.rt_lo;
  if (n_rt <= 0) return hipSuccess;
  const int group = p.Hq / p.Hkv;
  const int nh = pick_nh(group, D);
  const dim3 grid((unsigned)(n_rt * (p.Hq / nh))), block(256);
  TimedSpan span(timer, kKindFwd, stream);
  const bool sv = p.v_shared != nullptr;  // first-layer form: kernels that read chain V rows from the shared vector
  if (D == 64) {
    if (nh == 2) {
      if (sv) hipLaunchKernelGGL((fwd_kernel<64, 2, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((fwd_kernel<64, 2, false>), grid, block, 0, stream, p);
    } else {
      if (sv) hipLaunchKernelGGL((fwd_kernel<64, 1, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((fwd_kernel<64, 1, false>), grid, block, 0, stream, p);
    }
  } else {
    if (sv) return hipErrorInvalidValue;  // (D = 128 has no such instantiation: its callers expand V instead)
    hipLaunchKernelGGL((fwd_kernel<128, 1, false>), grid, block, 0, stream, p);
  }
  return span.finish();
}

hipError_t launch_bwd(const BwdParams& pin, int D, int key_lo, int a_hi, int acc_below, hipStream_t stream,
                      KernelTimer* timer) {
  BwdParams p = pin;
  const int n_rt = p.rt_hi - p.rt_lo;
  if (n_rt <= 0) return hipSuccess;
  // First-layer form.  The dQ kernel reads chain V rows from the shared vector at D = 64 only: at D = 128 it has
  // no registers to spare (that instantiation spilled three times as much and ran 25 % slower), so there the
  // caller passes an expanded V in `v` for it; the dK/dV kernel takes the shared vector at either size.
  const bool sv = p.v_shared != nullptr && D == 64, sv_dkdv = p.shared_dk_part != nullptr;
  {
    const dim3 grid((unsigned)(n_rt * p.Hq)), block(256);  // one query head per workgroup
    TimedSpan span(timer, kKindDq, stream);
    if (D == 64) {
      if (sv) hipLaunchKernelGGL((dq_pipe_kernel<64, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((dq_pipe_kernel<64, false>), grid, block, 0, stream, p);
    } else {
      hipLaunchKernelGGL((dq_kernel<128>), grid, block, 0, stream, p);
    }
    hipError_t e = span.finish();
    if (e != hipSuccess) return e;
  }
  // dK/dV runs over chunks of at most 64 row tiles (dense maps): within a chunk the key tiles below
  // its first anchor have equally long lists, which balances the workgroups the way the paper's
  // segments do; each chunk is followed by its own reduction, later chunks adding to what the
  // earlier ones wrote.
  const bool listed_map = p.tm.row_tok != nullptr;
  const int chunk = listed_map ? n_rt : 64;
  const int seg_rt_lo = p.rt_lo, seg_rt_hi = p.rt_hi;
  for (int c0 = seg_rt_lo; c0 < seg_rt_hi; c0 += chunk) {
    p.rt_lo = c0;
    p.rt_hi = c0 + chunk < seg_rt_hi ? c0 + chunk : seg_rt_hi;
    const bool partial = p.rt_lo != seg_rt_lo || p.rt_hi != seg_rt_hi;
    p.clip_rows = (pin.cropped || partial) ? 1 : 0;
    const int c_a_hi = listed_map || p.rt_hi * p.tm.A > a_hi ? a_hi : p.rt_hi * p.tm.A;
    const int c_acc = c0 == seg_rt_lo || acc_below == INT_MAX ? acc_below
                                                                : (acc_below > c0 * p.tm.A ? acc_below : c0 * p.tm.A);
    p.n_d0_tiles = (c_a_hi + kKeysPerTile - 1) / kKeysPerTile;  // depth-0 key tiles visible to rows < a_hi ...
    p.d0_tile_lo = key_lo / kKeysPerTile & ~1;                // ... from the (even) tile pair of the first visible key on
    p.n_d0_items = (p.n_d0_tiles - p.d0_tile_lo + 1) / 2 * p.Hq;  // key-tile pairs x query heads
    {
      // pairs wholly below the segment's first anchor see every row tile (equal lists); the others shrink
      const int n_pairs = (p.n_d0_tiles - p.d0_tile_lo + 1) / 2;
      const int equal = c_acc == INT_MAX ? 0 : (c_acc / kKeysPerTile - p.d0_tile_lo) / 2;
      const int shrinking = n_pairs - (equal > 0 ? equal : 0);
      constexpr int kPasses = 4;
      p.d0_step = (shrinking + kPasses - 1) / kPasses;
      if (p.d0_step < 2) p.d0_step = 2;
      p.d0_split = n_pairs - shrinking + p.d0_step;
      if (p.d0_split > n_pairs) p.d0_split = n_pairs;
    }
    const int n_chain_items = (p.rt_hi - p.rt_lo) * ((p.tm.n_csub + 1) / 2) * p.Hkv;
    {
      const dim3 grid((unsigned)(p.n_d0_items + n_chain_items));
      TimedSpan span(timer, kKindDkDv, stream);
      const bool listed = p.tm.row_tok != nullptr;
      auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, dim3(256), 0, stream, p); };
      if (D == 64) {
        if (listed) sv_dkdv ? go(dkdv_kernel<64, true, true>) : go(dkdv_kernel<64, true, false>);
        else sv_dkdv ? go(dkdv_kernel<64, false, true>) : go(dkdv_kernel<64, false, false>);
      } else {
        if (listed) sv_dkdv ? go(dkdv_kernel<128, true, true>) : go(dkdv_kernel<128, true, false>);
        else sv_dkdv ? go(dkdv_kernel<128, false, true>) : go(dkdv_kernel<128, false, false>);
      }
      hipError_t e = span.finish();
      if (e != hipSuccess) return e;
    }
    {
      const int key_first = p.d0_tile_lo * kKeysPerTile;
      const size_t n = 2 * (size_t)(c_a_hi - key_first) * p.Hkv * (D / 4);
      size_t blocks = (n + 255) / 256;
      if (blocks > 256 * 16) blocks = 256 * 16;
      const dim3 grid((unsigned)blocks), block(256);
      TimedSpan span(timer, kKindReduce, stream);
      if (D == 64) hipLaunchKernelGGL((reduce_partials_kernel<64>), grid, block, 0, stream, p, key_first, c_a_hi, c_acc);
      else hipLaunchKernelGGL((reduce_partials_kernel<128>), grid, block, 0, stream, p, key_first, c_a_hi, c_acc);
      hipError_t e = span.finish();
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

hipError_t launch_draft_decode(const DecodeParams& p, int D, hipStream_t stream) {
  // one computing wave per 32 query rows, plus the wave that copies
  const dim3 grid((unsigned)p.n_splits, (unsigned)p.Hkv, (unsigned)p.C), block((unsigned)((p.rows_pad / 32 + 1) * 64));
  // Long splits keep three tiles in flight per workgroup (4.4 against 4.1 TB/s on a batch that fills the
  // memory system); short ones - the serving shapes - are a microsecond faster with two buffers, which
  // let more workgroups share a CU.  D = 128 tiles are twice the size: two buffers.
  const bool deep = D == 64 && (p.max_pages + p.n_splits - 1) / p.n_splits > 16;
  if (D == 64) {
    if (deep) hipLaunchKernelGGL((draft_decode_kernel<64, 4>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((draft_decode_kernel<64, 2>), grid, block, 0, stream, p);
  } else {
    hipLaunchKernelGGL((draft_decode_kernel<128, 2>), grid, block, 0, stream, p);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t n = (size_t)p.C * p.Hkv * p.K * (p.Hq / p.Hkv) * (D / 4);
  size_t blocks = (n + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (D == 64) hipLaunchKernelGGL((draft_decode_combine_kernel<64>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL((draft_decode_combine_kernel<128>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_cast_bf16(const float* src, void* dst, size_t n, hipStream_t stream) {
  const size_t n4 = n / 4;
  if (n4 == 0) return hipSuccess;
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, (__bf16*)dst, n4);
  return hipGetLastError();
}

hipError_t measure_mfma_ceiling(hipStream_t stream, bool random_operands, float* tflops) {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  const int blocks = cus * 8, iters = 4000;
  float* out = nullptr;
  e = hipMalloc(&out, (size_t)blocks * 256 * sizeof(float));
  if (e != hipSuccess) return e;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    auto launch = [&] {
      if (random_operands) hipLaunchKernelGGL(mfma_ceiling_kernel<true>, dim3(blocks), dim3(256), 0, stream, out, iters);
      else hipLaunchKernelGGL(mfma_ceiling_kernel<false>, dim3(blocks), dim3(256), 0, stream, out, iters);
    };
    // warm-up: the clock settles over a few milliseconds of load
    for (int w = 0; w < 3; ++w) launch();
    (void)hipEventRecord(e0, stream);
    for (int w = 0; w < 3; ++w) launch();
    (void)hipEventRecord(e1, stream);
    e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) *tflops = (float)(3.0 * (double)blocks * 4 * iters * 4 * 32768.0 / ((double)ms * 1e9));
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(out);
  return e;
}

}  // namespace peagle
