// C-ABI entry points: host-side validation and the sequence-partition driver (Sec. 3.2 of the
// paper: one forward+backward pass per segment, dK/dV accumulated across segments in fp32).
#include <climits>
#include <cmath>
#include <mutex>

#include "attn_kernels.h"
#include "peagle.h"
#include "peagle_bench.h"
#include "tilemap.h"

using peagle::BwdParams;
using peagle::FwdParams;
using peagle::SegRange;

static_assert(PEAGLE_NUM_KERNEL_KINDS == peagle::kNumKinds, "public and internal kernel kinds differ");

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
  size_t delta_off, nlse_off, dk_off, dv_off, total;
  int L64;
};

// Stored tokens of the call: L*K for a dense map, the kept positions for a sampled one.
size_t tokens_of(const peagle_tilemap_t* tm, const peagle_shape_t* s) {
  return tm->sampled ? (size_t)tm->T_tokens : (size_t)s->L * s->K;
}

WsLayout ws_layout(const peagle_tilemap_t* tm, const peagle_shape_t* s) {
  WsLayout w;
  w.L64 = (s->L + 63) / 64 * 64;
  const size_t T = tokens_of(tm, s);
  const size_t part = (size_t)s->Hq * w.L64 * s->D * sizeof(float);
  w.delta_off = 0;
  w.nlse_off = align256(T * s->Hq * sizeof(float));
  w.dk_off = w.nlse_off + align256(T * s->Hq * sizeof(float));
  w.dv_off = w.dk_off + align256(part);
  w.total = w.dv_off + align256(part);
  return w;
}

int check_shape(const peagle_tilemap_t* tm, const peagle_shape_t* s) {
  if (!tm || !s) return PEAGLE_ENULL;
  if (s->L < 1 || s->Hq < 1 || s->Hkv < 1 || s->K < 1) return PEAGLE_EINVAL;
  if (s->Hq % s->Hkv != 0) return PEAGLE_EINVAL;
  if (!(s->scale > 0.f) || !std::isfinite(s->scale)) return PEAGLE_EINVAL;
  if (s->layout != PEAGLE_LAYOUT_DEPTH_MAJOR) return PEAGLE_EUNSUPPORTED;
  if (s->D != 64 && s->D != 128) return PEAGLE_EUNSUPPORTED;
  if (s->K != tm->K || s->L > tm->L_max) return PEAGLE_ESHAPE;
  if (tm->sampled && s->L != tm->L_max) return PEAGLE_ESHAPE;  // a sampled map serves its own sequence only
  return PEAGLE_OK;
}

// First-layer form of the step (null members: the ordinary step)
struct SharedForm {
  const void* v_shared = nullptr;  // [Hkv, D]: the value row of every chain key
  float* dk_part = nullptr;        // per-wave sums of the chain keys' dK / dV, see BwdParams
  float* dv_part = nullptr;
  bool fwd_reads_v_tensor = false;  // `v` is a full [T, Hkv, D] tensor: the forward does not need v_shared
};

FwdParams make_fwd(const peagle_tilemap_t* tm, const peagle_shape_t* s, const SegRange& sr, const void* q,
                   const void* k, const void* v, void* o, float* lse, const SharedForm& sf = SharedForm()) {
  FwdParams p{};
  p.v_shared = sf.fwd_reads_v_tensor ? nullptr : (const __bf16*)sf.v_shared;
  p.q = (const __bf16*)q;
  p.k = (const __bf16*)k;
  p.v = (const __bf16*)v;
  p.o = (__bf16*)o;
  p.lse = lse;
  p.tm = tm->dview;
  p.L = s->L;
  p.T = (int)tokens_of(tm, s);
  p.Hq = s->Hq;
  p.Hkv = s->Hkv;
  p.rt_lo = sr.rt_lo;
  p.rt_hi = sr.rt_hi;
  p.c_log2 = s->scale * 1.4426950408889634f;
  return p;
}

BwdParams make_bwd(const peagle_tilemap_t* tm, const peagle_shape_t* s, const SegRange& sr, const void* q,
                   const void* k, const void* v, const void* o, const void* d_o, const float* lse, void* dq,
                   float* dk_acc, float* dv_acc, void* workspace, int chain_accumulate,
                   const float* rope_table = nullptr, const SharedForm& sf = SharedForm()) {
  const WsLayout w = ws_layout(tm, s);
  BwdParams p{};
  p.v_shared = (const __bf16*)sf.v_shared;
  p.shared_dk_part = sf.dk_part;
  p.shared_dv_part = sf.dv_part;
  p.q = (const __bf16*)q;
  p.k = (const __bf16*)k;
  p.v = (const __bf16*)v;
  p.o = (const __bf16*)o;
  p.d_o = (const __bf16*)d_o;
  p.lse = lse;
  p.dq = (__bf16*)dq;
  p.dk_acc = dk_acc;
  p.dv_acc = dv_acc;
  p.delta = (float*)((char*)workspace + w.delta_off);
  p.nlse = (float*)((char*)workspace + w.nlse_off);
  p.dk_part = (float*)((char*)workspace + w.dk_off);
  p.dv_part = (float*)((char*)workspace + w.dv_off);
  p.tm = tm->dview;
  p.L = s->L;
  p.T = (int)tokens_of(tm, s);
  p.Hq = s->Hq;
  p.Hkv = s->Hkv;
  p.L64 = w.L64;
  p.rt_lo = sr.rt_lo;
  p.rt_hi = sr.rt_hi;
  p.s_lo = sr.s_lo;
  p.s_hi = sr.s_hi;
  p.cropped = sr.cropped;
  p.fast_rows = (size_t)p.T * s->Hq * s->D * 2 < ((size_t)1 << 32) ? 1 : 0;
  p.chain_accumulate = chain_accumulate;
  p.c_log2 = s->scale * 1.4426950408889634f;
  p.scale = s->scale;
  p.rope_table = rope_table;
  return p;
}

// Rotary embedding: positions the table must cover, and where the rotated copies of Q and K live
// behind the attention workspace.
int32_t rope_positions(const peagle_tilemap_t* tm, int32_t L) {
  return tm->sampled ? tm->max_posid + 1 : L + tm->K - 1;
}
struct RopeWs {
  size_t q_off, k_off, total;
};
RopeWs rope_ws(const peagle_tilemap_t* tm, const peagle_shape_t* s) {
  RopeWs w;
  const size_t T = tokens_of(tm, s);
  w.q_off = ws_layout(tm, s).total;
  w.k_off = w.q_off + align256(T * s->Hq * s->D * 2);
  w.total = w.k_off + align256(T * s->Hkv * s->D * 2);
  return w;
}

}  // namespace

extern "C" size_t peagle_workspace_bytes(const peagle_tilemap_t* tm, const peagle_shape_t* shape) {
  if (check_shape(tm, shape) != PEAGLE_OK) return 0;
  return ws_layout(tm, shape).total;
}

extern "C" int peagle_attn_fwd(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg, const void* q,
                               const void* k, const void* v, void* o, float* lse, void* stream) {
  int rc = check_shape(tm, shape);
  if (rc != PEAGLE_OK) return rc;
  if (!q || !k || !v || !o || !lse) return PEAGLE_ENULL;
  SegRange sr;
  rc = peagle::resolve_segment(tm, shape->L, seg, &sr);
  if (rc != PEAGLE_OK) return rc;
  if (tm->device < 0) return PEAGLE_ENODEVICE;
  const FwdParams p = make_fwd(tm, shape, sr, q, k, v, o, lse);
  return peagle::launch_fwd(p, shape->D, (hipStream_t)stream) == hipSuccess ? PEAGLE_OK : PEAGLE_EHIP;
}

extern "C" int peagle_attn_bwd(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg, const void* q,
                               const void* k, const void* v, const void* o, const void* d_o, const float* lse,
                               void* dq, float* dk_acc, float* dv_acc, int32_t accumulate, void* workspace,
                               size_t ws_bytes, void* stream) {
  int rc = check_shape(tm, shape);
  if (rc != PEAGLE_OK) return rc;
  if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk_acc || !dv_acc) return PEAGLE_ENULL;
  if (accumulate != 0 && accumulate != 1) return PEAGLE_EINVAL;
  SegRange sr;
  rc = peagle::resolve_segment(tm, shape->L, seg, &sr);
  if (rc != PEAGLE_OK) return rc;
  if (!workspace || ws_bytes < ws_layout(tm, shape).total) return PEAGLE_EWORKSPACE;
  if (tm->device < 0) return PEAGLE_ENODEVICE;
  const BwdParams p = make_bwd(tm, shape, sr, q, k, v, o, d_o, lse, dq, dk_acc, dv_acc, workspace, accumulate);
  const int acc_below = accumulate ? INT_MAX : 0;
  return peagle::launch_bwd(p, shape->D, sr.key_lo, sr.a_hi, acc_below, (hipStream_t)stream) == hipSuccess ? PEAGLE_OK
                                                                                                   : PEAGLE_EHIP;
}

static int step_impl(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg_begin, int32_t seg_end,
                     const void* q, const void* k, const void* v, const void* d_o, void* o, float* lse, void* dq,
                     float* dk_acc, float* dv_acc, void* dk_bf16, void* dv_bf16, void* workspace, size_t ws_bytes,
                     void* stream, peagle::KernelTimer* timer, const float* rope_table = nullptr,
                     int32_t rope_n_pos = 0, bool inputs_rotated = false, const SharedForm& sf = SharedForm()) {
  int rc = check_shape(tm, shape);
  if (rc != PEAGLE_OK) return rc;
  if (!q || !k || !v || !d_o || !o || !lse || !dq || !dk_acc || !dv_acc) return PEAGLE_ENULL;
  if (seg_begin < 0 || seg_end > tm->S || seg_begin > seg_end) return PEAGLE_EINVAL;
  const size_t ws_need = rope_table ? rope_ws(tm, shape).total : ws_layout(tm, shape).total;
  if (!workspace || ws_bytes < ws_need) return PEAGLE_EWORKSPACE;
  if (rope_table && rope_n_pos < rope_positions(tm, shape->L)) return PEAGLE_ESHAPE;
  if (tm->device < 0) return PEAGLE_ENODEVICE;
  hipStream_t st = (hipStream_t)stream;
  if (rope_table && !inputs_rotated) {
    // Q and K arrive unrotated: the attention runs on rotated copies kept behind the workspace
    const RopeWs rw = rope_ws(tm, shape);
    void* q_rot = (char*)workspace + rw.q_off;
    void* k_rot = (char*)workspace + rw.k_off;
    const int T = (int)tokens_of(tm, shape);
    if (peagle::launch_rope_rotate(q, q_rot, shape->Hq, T, shape->D, tm->dview, shape->L, rope_table, false, st,
                                   timer) != hipSuccess)
      return PEAGLE_EHIP;
    if (peagle::launch_rope_rotate(k, k_rot, shape->Hkv, T, shape->D, tm->dview, shape->L, rope_table, false, st,
                                   timer) != hipSuccess)
      return PEAGLE_EHIP;
    q = q_rot;
    k = k_rot;
  }
  for (int32_t s = seg_begin; s < seg_end; ++s) {
    SegRange sr;
    rc = peagle::resolve_segment(tm, shape->L, s, &sr);
    if (rc != PEAGLE_OK) return rc;
    if (sr.a_lo >= sr.a_hi) continue;  // segment lies beyond the cropped length
    const FwdParams fp = make_fwd(tm, shape, sr, q, k, v, o, lse, sf);
    if (peagle::launch_fwd(fp, shape->D, st, timer) != hipSuccess) return PEAGLE_EHIP;
    // Depth-0 keys below the segment start already hold earlier segments' sums: add to them.
    // Keys first seen by this segment (its own depth-0 range and its chains) are overwritten.
    const BwdParams bp = make_bwd(tm, shape, sr, q, k, v, o, d_o, lse, dq, dk_acc, dv_acc, workspace, 0, rope_table, sf);
    if (peagle::launch_bwd(bp, shape->D, sr.key_lo, sr.a_hi, sr.a_lo, st, timer) != hipSuccess) return PEAGLE_EHIP;
  }
  if (seg_end == tm->S || tm->seg_bounds[seg_end] >= shape->L) {
    const size_t n = tokens_of(tm, shape) * shape->Hkv * shape->D;
    if (dk_bf16 && peagle::launch_cast_bf16(dk_acc, dk_bf16, n, st) != hipSuccess) return PEAGLE_EHIP;
    if (dv_bf16 && peagle::launch_cast_bf16(dv_acc, dv_bf16, n, st) != hipSuccess) return PEAGLE_EHIP;
  }
  return PEAGLE_OK;
}

extern "C" int peagle_attn_step_partitioned(const peagle_tilemap_t* tm, const peagle_shape_t* shape,
                                            int32_t seg_begin, int32_t seg_end, const void* q, const void* k,
                                            const void* v, const void* d_o, void* o, float* lse, void* dq,
                                            float* dk_acc, float* dv_acc, void* dk_bf16, void* dv_bf16,
                                            void* workspace, size_t ws_bytes, void* stream) {
  return step_impl(tm, shape, seg_begin, seg_end, q, k, v, d_o, o, lse, dq, dk_acc, dv_acc, dk_bf16, dv_bf16,
                   workspace, ws_bytes, stream, nullptr);
}

extern "C" int peagle_attn_step_profiled(const peagle_tilemap_t* tm, const peagle_shape_t* shape, int32_t seg_begin,
                                         int32_t seg_end, const void* q, const void* k, const void* v,
                                         const void* d_o, void* o, float* lse, void* dq, float* dk_acc,
                                         float* dv_acc, void* workspace, size_t ws_bytes, void* stream,
                                         peagle_profile_t* profile) {
  if (!profile) return PEAGLE_ENULL;
  for (int i = 0; i < PEAGLE_NUM_KERNEL_KINDS; ++i) {
    profile->ms[i] = 0.f;
    profile->launches[i] = 0;
  }
  peagle::KernelTimer timer;
  int rc = step_impl(tm, shape, seg_begin, seg_end, q, k, v, d_o, o, lse, dq, dk_acc, dv_acc, nullptr, nullptr,
                     workspace, ws_bytes, stream, &timer);
  if (rc != PEAGLE_OK) return rc;
  return timer.collect(profile->ms, profile->launches) == hipSuccess ? PEAGLE_OK : PEAGLE_EHIP;
}

extern "C" int32_t peagle_rope_positions(const peagle_tilemap_t* tm, int32_t L) {
  if (!tm || L < 1 || L > tm->L_max || (tm->sampled && L != tm->L_max)) return -1;
  return rope_positions(tm, L);
}

extern "C" int peagle_rope_position_ids(const peagle_tilemap_t* tm, int32_t L, int32_t* pos_out) {
  if (!tm || !pos_out) return PEAGLE_ENULL;
  if (L < 1 || L > tm->L_max || (tm->sampled && L != tm->L_max)) return PEAGLE_ESHAPE;
  if (tm->sampled) {
    for (size_t t = 0; t < tm->tok_posid.size(); ++t) pos_out[t] = tm->tok_posid[t];
  } else {
    for (int32_t d = 0; d < tm->K; ++d)
      for (int32_t i = 0; i < L; ++i) pos_out[(size_t)d * L + i] = i + d;
  }
  return PEAGLE_OK;
}

extern "C" int peagle_rope_table(float base, int32_t D, int32_t n_pos, float* table, void* stream) {
  if (!table) return PEAGLE_ENULL;
  if (!(base > 1.f) || !std::isfinite(base) || n_pos < 1) return PEAGLE_EINVAL;
  if (D != 64 && D != 128) return PEAGLE_EUNSUPPORTED;
  return peagle::launch_rope_table((double)base, D, n_pos, table, (hipStream_t)stream) == hipSuccess ? PEAGLE_OK
                                                                                                      : PEAGLE_EHIP;
}

extern "C" int peagle_rope_rotate(const peagle_tilemap_t* tm, const peagle_shape_t* shape, const void* x, int32_t H,
                                  const float* rope_table, int32_t n_pos, int32_t inverse, void* out, void* stream) {
  int rc = check_shape(tm, shape);
  if (rc != PEAGLE_OK) return rc;
  if (!x || !out || !rope_table) return PEAGLE_ENULL;
  if (H < 1 || (inverse != 0 && inverse != 1)) return PEAGLE_EINVAL;
  if (n_pos < rope_positions(tm, shape->L)) return PEAGLE_ESHAPE;
  if (tm->device < 0) return PEAGLE_ENODEVICE;
  return peagle::launch_rope_rotate(x, out, H, (int)tokens_of(tm, shape), shape->D, tm->dview, shape->L, rope_table,
                                    inverse != 0, (hipStream_t)stream) == hipSuccess
             ? PEAGLE_OK
             : PEAGLE_EHIP;
}

extern "C" size_t peagle_rope_workspace_bytes(const peagle_tilemap_t* tm, const peagle_shape_t* shape) {
  if (check_shape(tm, shape) != PEAGLE_OK) return 0;
  return rope_ws(tm, shape).total;
}

extern "C" int peagle_attn_step_partitioned_rope(const peagle_tilemap_t* tm, const peagle_shape_t* shape,
                                                 int32_t seg_begin, int32_t seg_end, const void* q, const void* k,
                                                 const void* v, const void* d_o, const float* rope_table,
                                                 int32_t n_pos, void* o, float* lse, void* dq, float* dk_acc,
                                                 float* dv_acc, void* dk_bf16, void* dv_bf16, void* workspace,
                                                 size_t ws_bytes, void* stream) {
  if (!rope_table) return PEAGLE_ENULL;
  return step_impl(tm, shape, seg_begin, seg_end, q, k, v, d_o, o, lse, dq, dk_acc, dv_acc, dk_bf16, dv_bf16,
                   workspace, ws_bytes, stream, nullptr, rope_table, n_pos);
}

namespace {

// Workspace of the first-layer form: the rotary workspace (rotated Q, expanded and rotated K), the per-wave sums
// of the chain keys' dK / dV (one row of Hkv x D per wave of every chain-tile workgroup) and, at D = 128 only, an
// expanded V (the forward and dQ kernels of that size do not read chain V rows from the shared vector).
struct SharedWs {
  size_t pk_off, pv_off, v_off, total;
  int32_t part_rows;
};
SharedWs shared_ws(const peagle_tilemap_t* tm, const peagle_shape_t* s) {
  SharedWs w;
  const size_t cols = (size_t)s->Hkv * s->D;
  w.part_rows = tm->n_row_tiles * ((tm->n_csub + 1) / 2) * 4;
  w.pk_off = rope_ws(tm, s).total;
  w.pv_off = w.pk_off + align256((size_t)w.part_rows * cols * sizeof(float));
  w.v_off = w.pv_off + align256((size_t)w.part_rows * cols * sizeof(float));
  w.total = w.v_off + (s->D == 64 ? 0 : align256(tokens_of(tm, s) * cols * 2));
  return w;
}

}  // namespace

extern "C" size_t peagle_rope_shared_workspace_bytes(const peagle_tilemap_t* tm, const peagle_shape_t* shape) {
  if (check_shape(tm, shape) != PEAGLE_OK) return 0;
  return shared_ws(tm, shape).total;
}

extern "C" int peagle_attn_step_rope_shared(const peagle_tilemap_t* tm, const peagle_shape_t* shape, const void* q,
                                            const void* k0, const void* k_shared, const void* v0,
                                            const void* v_shared, const void* d_o, const float* rope_table,
                                            int32_t n_pos, void* o, float* lse, void* dq, float* dk0, float* dv0,
                                            float* dk_shared, float* dv_shared, void* workspace, size_t ws_bytes,
                                            void* stream) {
  int rc = check_shape(tm, shape);
  if (rc != PEAGLE_OK) return rc;
  if (!q || !k0 || !k_shared || !v0 || !v_shared || !d_o || !rope_table || !o || !lse || !dq || !dk0 || !dv0 ||
      !dk_shared || !dv_shared)
    return PEAGLE_ENULL;
  if (n_pos < rope_positions(tm, shape->L)) return PEAGLE_ESHAPE;
  const SharedWs sw = shared_ws(tm, shape);
  if (!workspace || ws_bytes < sw.total) return PEAGLE_EWORKSPACE;
  if (tm->device < 0) return PEAGLE_ENODEVICE;
  hipStream_t st = (hipStream_t)stream;
  const RopeWs rw = rope_ws(tm, shape);
  const int T = (int)tokens_of(tm, shape), L0 = shape->L;  // the depth-0 positions are the first L stored tokens
  char* ws = (char*)workspace;
  void* q_rot = ws + rw.q_off;
  void* k_rot = ws + rw.k_off;
  if (peagle::launch_rope_rotate(q, q_rot, shape->Hq, T, shape->D, tm->dview, shape->L, rope_table, false, st) !=
      hipSuccess)
    return PEAGLE_EHIP;
  // K: the depth-0 rows and, for every chain token, the shared vector turned to that token's position
  if (peagle::launch_expand_shared(k0, k_shared, k_rot, shape->Hkv, T, L0, shape->D, tm->dview, shape->L, rope_table,
                                   st) != hipSuccess)
    return PEAGLE_EHIP;
  // V is not expanded: the kernels take every chain key's value row from v_shared, and v0 holds exactly the rows
  // of the depth-0 tokens (the first L0 of the stored order).  Likewise dK / dV: the depth-0 keys' gradients go
  // straight to the caller's dk0 / dv0 (the first L0 rows are all the kernels write there in this form), the
  // chain keys' come out as per-wave sums.
  SharedForm sf;
  sf.v_shared = v_shared;
  sf.dk_part = (float*)(ws + sw.pk_off);
  sf.dv_part = (float*)(ws + sw.pv_off);
  const void* v_arg = v0;
  if (shape->D != 64) {
    // (this size's forward and dQ kernels read every V row from a tensor: expand V for them)
    void* v_full = ws + sw.v_off;
    if (peagle::launch_expand_shared(v0, v_shared, v_full, shape->Hkv, T, L0, shape->D, tm->dview, shape->L, nullptr,
                                     st) != hipSuccess)
      return PEAGLE_EHIP;
    v_arg = v_full;
    sf.fwd_reads_v_tensor = true;
  }
  rc = step_impl(tm, shape, 0, tm->S, q_rot, k_rot, v_arg, d_o, o, lse, dq, dk0, dv0, nullptr, nullptr, workspace,
                 ws_bytes, stream, nullptr, rope_table, n_pos, /*inputs_rotated=*/true, sf);
  if (rc != PEAGLE_OK) return rc;
  SegRange whole;
  rc = peagle::resolve_segment(tm, shape->L, -1, &whole);
  if (rc != PEAGLE_OK) return rc;
  const int rows = whole.rt_hi * ((tm->n_csub + 1) / 2) * 4;  // rows written by a length-L step
  return peagle::launch_shared_grads(sf.dk_part, sf.dv_part, rows, dk_shared, dv_shared, shape->Hkv * shape->D,
                                     st) == hipSuccess
             ? PEAGLE_OK
             : PEAGLE_EHIP;
}

extern "C" int peagle_attn_step_rope_profiled(const peagle_tilemap_t* tm, const peagle_shape_t* shape,
                                              int32_t seg_begin, int32_t seg_end, const void* q, const void* k,
                                              const void* v, const void* d_o, const float* rope_table, int32_t n_pos,
                                              void* o, float* lse, void* dq, float* dk_acc, float* dv_acc,
                                              void* workspace, size_t ws_bytes, void* stream,
                                              peagle_profile_t* profile) {
  if (!profile || !rope_table) return PEAGLE_ENULL;
  for (int i = 0; i < PEAGLE_NUM_KERNEL_KINDS; ++i) {
    profile->ms[i] = 0.f;
    profile->launches[i] = 0;
  }
  peagle::KernelTimer timer;
  int rc = step_impl(tm, shape, seg_begin, seg_end, q, k, v, d_o, o, lse, dq, dk_acc, dv_acc, nullptr, nullptr,
                     workspace, ws_bytes, stream, &timer, rope_table, n_pos);
  if (rc != PEAGLE_OK) return rc;
  return timer.collect(profile->ms, profile->launches) == hipSuccess ? PEAGLE_OK : PEAGLE_EHIP;
}

namespace {

int check_decode(const peagle_decode_shape_t* s) {
  if (!s) return PEAGLE_ENULL;
  if (s->C < 1 || s->K < 1 || s->Hq < 1 || s->Hkv < 1 || s->n_pages < 1 || s->max_pages < 1) return PEAGLE_EINVAL;
  if (s->Hq % s->Hkv != 0) return PEAGLE_EINVAL;
  if (!(s->scale > 0.f) || !std::isfinite(s->scale)) return PEAGLE_EINVAL;
  if (s->D != 64 && s->D != 128) return PEAGLE_EUNSUPPORTED;
  if ((int64_t)s->K * (s->Hq / s->Hkv) > peagle::kRowsPerTile || s->K > peagle::kKeysPerTile) return PEAGLE_EUNSUPPORTED;
  if (s->C > 65535 || s->Hkv > 65535) return PEAGLE_EUNSUPPORTED;  // grid dimensions
  if (s->max_pages > (1 << 24)) return PEAGLE_EUNSUPPORTED;          // 64 * max_pages tokens must fit an int
  return PEAGLE_OK;
}

// Pieces each request's context is cut into: enough workgroups to cover the chip a few times over,
// but at least four pages per piece so that the partial records stay small next to the cache read.
int decode_splits(const peagle_decode_shape_t* s) {
  const int64_t want = (1024 + (int64_t)s->C * s->Hkv - 1) / ((int64_t)s->C * s->Hkv);
  const int64_t most = (s->max_pages + 3) / 4;
  int64_t n = want < most ? want : most;
  if (n > 32) n = 32;
  return (int)(n < 1 ? 1 : n);
}

struct DecodeWs {
  size_t o_off, ml_off, total;
  int rows_pad, n_splits;
};
DecodeWs decode_ws(const peagle_decode_shape_t* s) {
  DecodeWs w;
  w.n_splits = decode_splits(s);
  w.rows_pad = (s->K * (s->Hq / s->Hkv) + 31) / 32 * 32;
  const size_t recs = (size_t)s->C * s->Hkv * w.n_splits;
  w.o_off = 0;
  w.ml_off = align256(recs * w.rows_pad * s->D * sizeof(float));
  w.total = w.ml_off + align256(recs * 3 * w.rows_pad * sizeof(float));
  return w;
}

}  // namespace

extern "C" int32_t peagle_draft_decode_splits(const peagle_decode_shape_t* shape) {
  return check_decode(shape) == PEAGLE_OK ? decode_splits(shape) : -1;
}

extern "C" size_t peagle_draft_decode_workspace_bytes(const peagle_decode_shape_t* shape) {
  return check_decode(shape) == PEAGLE_OK ? decode_ws(shape).total : 0;
}

namespace {

int decode_impl(const peagle_decode_shape_t* shape, const DecodeWs& w, const void* q_new, const void* k_new,
                const void* v_new, const void* k_pages, const void* v_pages, const int32_t* block_table,
                const int32_t* ctx_len, void* o, float* lse, int32_t* status, void* workspace, void* stream) {
  peagle::DecodeParams p{};
  p.q_new = (const __bf16*)q_new;
  p.k_new = (const __bf16*)k_new;
  p.v_new = (const __bf16*)v_new;
  p.k_pages = (const __bf16*)k_pages;
  p.v_pages = (const __bf16*)v_pages;
  p.block_table = block_table;
  p.ctx_len = ctx_len;
  p.o = (__bf16*)o;
  p.lse = lse;
  p.status = status;
  p.part_o = (float*)((char*)workspace + w.o_off);
  p.part_ml = (float*)((char*)workspace + w.ml_off);
  p.C = shape->C;
  p.K = shape->K;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.n_pages = shape->n_pages;
  p.max_pages = shape->max_pages;
  p.n_splits = w.n_splits;
  p.rows_pad = w.rows_pad;
  p.c_log2 = shape->scale * 1.4426950408889634f;
  return peagle::launch_draft_decode(p, shape->D, (hipStream_t)stream) == hipSuccess ? PEAGLE_OK : PEAGLE_EHIP;
}

}  // namespace

extern "C" int peagle_draft_decode(const peagle_decode_shape_t* shape, const void* q_new, const void* k_new,
                                   const void* v_new, const void* k_pages, const void* v_pages,
                                   const int32_t* block_table, const int32_t* ctx_len, void* o, float* lse,
                                   int32_t* status, void* workspace, size_t ws_bytes, void* stream) {
  const int rc = check_decode(shape);
  if (rc != PEAGLE_OK) return rc;
  if (!q_new || !k_new || !v_new || !k_pages || !v_pages || !block_table || !ctx_len || !o || !lse) return PEAGLE_ENULL;
  const DecodeWs w = decode_ws(shape);
  if (!workspace || ws_bytes < w.total) return PEAGLE_EWORKSPACE;
  return decode_impl(shape, w, q_new, k_new, v_new, k_pages, v_pages, block_table, ctx_len, o, lse, status, workspace,
                     stream);
}

// Partial records of peagle_draft_decode_static: one array per GPU, held by the loaded library until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the device address
// it yields (one per device, looked up once with that device current) is what kernels are given.
static __device__ __align__(256) unsigned char scratch[PEAGLE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return PEAGLE_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return PEAGLE_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PEAGLE_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PEAGLE_OK;
}

}  // namespace

extern "C" int peagle_draft_decode_static(const peagle_decode_shape_t* shape, const void* q_new, const void* k_new,
                                          const void* v_new, const void* k_pages, const void* v_pages,
                                          const int32_t* block_table, const int32_t* ctx_len, void* o, float* lse,
                                          int32_t* status, void* stream) {
  const int rc = check_decode(shape);
  if (rc != PEAGLE_OK) return rc;
  if (!q_new || !k_new || !v_new || !k_pages || !v_pages || !block_table || !ctx_len || !o || !lse) return PEAGLE_ENULL;
  const DecodeWs w = decode_ws(shape);
  if (w.total > (size_t)PEAGLE_STATIC_SCRATCH_BYTES) return PEAGLE_EWORKSPACE;
  void* ws = nullptr;
  const int src = static_scratch(&ws);
  if (src != PEAGLE_OK) return src;
  // Every partial record the merge reads is written by this call's first launch: nothing has to start at zero.
  return decode_impl(shape, w, q_new, k_new, v_new, k_pages, v_pages, block_table, ctx_len, o, lse, status, ws, stream);
}

extern "C" int peagle_measure_mfma_ceiling(void* stream, float* tflops) {
  if (!tflops) return PEAGLE_ENULL;
  *tflops = 0.f;
  return peagle::measure_mfma_ceiling((hipStream_t)stream, false, tflops) == hipSuccess ? PEAGLE_OK : PEAGLE_EHIP;
}

extern "C" int peagle_measure_mfma_ceiling_random(void* stream, float* tflops) {
  if (!tflops) return PEAGLE_ENULL;
  *tflops = 0.f;
  return peagle::measure_mfma_ceiling((hipStream_t)stream, true, tflops) == hipSuccess ? PEAGLE_OK : PEAGLE_EHIP;
}

extern "C" int peagle_device_info(int32_t* compute_units, int32_t* clock_khz) {
  if (!compute_units || !clock_khz) return PEAGLE_ENULL;
  int dev = 0, cus = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) return PEAGLE_EHIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return PEAGLE_EHIP;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess) return PEAGLE_EHIP;
  *compute_units = cus;
  *clock_khz = khz;
  return PEAGLE_OK;
}
