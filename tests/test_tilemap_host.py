"""Host-only tests (no GPU): the C-ABI library loads and exports every declared symbol, argument
validation returns the documented codes, and the tile map expands bit-exactly to the oracle's
element mask (parallel-prediction mask of Sec. 3; crop invariance of Sec. 3.1; segments of Sec. 3.2)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2602_01469_amd as pe
from paper_2602_01469_amd import binding
from oracle import peagle_oracle as orc
from peagle_inputs import CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _expanded(tm, L, K, seg, rows):
    """Element mask rows (bool [len(rows), T]) from the tile map, for sorted contiguous row blocks."""
    T = L * K
    out = np.zeros((len(rows), T), dtype=bool)
    rows = np.asarray(rows)
    # contiguous runs
    starts = np.flatnonzero(np.diff(np.concatenate([[-2], rows])) != 1)
    ends = np.concatenate([starts[1:], [len(rows)]])
    for s, e in zip(starts, ends):
        bits = tm.expand_rows(L, seg, int(rows[s]), int(rows[e - 1]) + 1)
        out[s:e] = np.unpackbits(bits, axis=1, bitorder="little")[:, :T].astype(bool)
    return out


def test_library_exports_every_declared_symbol():
    lib = pe.load_library()
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("peagle.h", "peagle_bench.h"))
    declared = set(re.findall(r"\b(peagle_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("L,K", [(1, 1), (1, 8), (17, 4), (128, 4), (100, 8), (50, 3), (300, 1), (129, 5), (70, 16),
                                 (40, 128), (333, 7)])
def test_tilemap_expands_to_oracle_mask_bit_exact(L, K):
    tm = pe.peagle_build_tilemap(L, K, None, device=-1)
    T = L * K
    got = _expanded(tm, L, K, -1, np.arange(T))
    assert np.array_equal(got, orc.element_mask(L, K))
    inf = tm.info()
    assert inf["anchors_per_row_tile"] == 128 // K
    assert inf["n_masks"] <= 2 * 64 + inf["n_chain_sub_tiles"]   # O(1): one per residue of the tile offset


@pytest.mark.parametrize("L_max,L,K", [(256, 219, 8), (256, 1, 8), (256, 64, 4), (500, 333, 3), (512, 500, 1)])
def test_crop_is_prefix_view(L_max, L, K):
    """Per-example mask = crop of the maximum-length mask (Sec. 3.1): same tile map, shorter L."""
    tm = pe.peagle_build_tilemap(L_max, K, None, device=-1)
    got = _expanded(tm, L, K, -1, np.arange(L * K))
    assert np.array_equal(got, orc.element_mask(L, K))


def test_segments_partition_rows_and_union_is_full_mask():
    L, K = 256, 8
    bounds = [0, 64, 128, 256]
    tm = pe.peagle_build_tilemap(L, K, bounds, device=-1)
    T = L * K
    full = orc.element_mask(L, K)
    union = np.zeros((T, T), dtype=bool)
    for s in range(3):
        got = _expanded(tm, L, K, s, np.arange(T))
        rows = orc.segment_rows(L, K, bounds[s], bounds[s + 1])
        cols = orc.segment_keys(L, K, bounds[s], bounds[s + 1])
        other = np.setdiff1d(np.arange(T), rows)
        assert not got[other].any()                       # rows outside the segment are untouched
        assert np.array_equal(got[rows], full[rows])      # its rows carry their full visible set
        assert not got[:, np.setdiff1d(np.arange(T), cols)].any()  # only cumulative depth-0 + own chains
        assert not (union & got).any()
        union |= got
    assert np.array_equal(union, full)


def test_segments_with_crop():
    L_max, L, K = 256, 150, 8
    tm = pe.peagle_build_tilemap(L_max, K, [0, 64, 128, 256], device=-1)
    full = orc.element_mask(L, K)
    union = np.zeros_like(full)
    for s in range(3):
        union |= _expanded(tm, L, K, s, np.arange(L * K))
    assert np.array_equal(union, full)


@pytest.mark.parametrize("name", ["c2_gptoss", "c3_median", "c4_p90", "c5_p99"])
def test_tilemap_full_size_configs_sampled_rows(name):
    """Full-size tile maps against the oracle mask on whole row tiles sampled over the sequence
    (first, last, around every segment boundary, random), plus closed-form pair counts."""
    cfg = CONFIGS[name]
    b = cfg.seg_bounds()
    tm = pe.peagle_build_tilemap(cfg.L, cfg.K, b, device=-1)
    inf = tm.info()
    A = inf["anchors_per_row_tile"]
    rng = np.random.default_rng(0)
    anchors = {0, cfg.L - A, (cfg.L // 2 // A) * A}
    for x in b[1:-1]:
        anchors |= {int(x) - A, int(x)}
    anchors |= {int(a) * A for a in rng.integers(0, cfg.L // A, size=4)}
    for a0 in sorted(anchors):
        rows = np.concatenate([d * cfg.L + np.arange(a0, min(a0 + A, cfg.L)) for d in range(cfg.K)])
        rows.sort()
        got = _expanded(tm, cfg.L, cfg.K, -1, rows)
        ref = orc.element_mask(cfg.L, cfg.K, rows=rows)
        assert np.array_equal(got, ref), (name, a0)
    n_rt, n_d0 = inf["n_row_tiles"], inf["n_depth0_key_tiles"]
    assert n_rt == -(-cfg.L // A) and n_d0 == -(-cfg.L // 64)
    # closed forms: key tile c is full for row tile R iff 64c+63 <= R*A; each row tile adds the
    # depth-0 tile(s) its anchors straddle and its chain sub-tiles as partial pairs
    assert inf["n_full"] == sum((R * A + 1) // 64 for R in range(n_rt))
    n_partial_d0 = sum(min((R * A + A - 1) // 64, n_d0 - 1) - (R * A + 1) // 64 + 1 for R in range(n_rt))
    assert inf["n_partial"] == n_partial_d0 + n_rt * inf["n_chain_sub_tiles"]
    assert inf["n_masks"] <= 64 // A + 1 + inf["n_chain_sub_tiles"] + 2


def test_mask_pool_does_not_grow_with_length():
    """Position invariance (Sec. 3.1) at tile level: the pool of distinct bitmasks is the same for any length."""
    small = pe.peagle_build_tilemap(1024, 8, None, device=-1).info()["n_masks"]
    large = pe.peagle_build_tilemap(20480, 8, None, device=-1).info()["n_masks"]
    assert small == large == 6


def test_classes_map_small():
    L, K = 128, 4
    tm = pe.peagle_build_tilemap(L, K, None, device=-1)
    cls = tm.classes()
    inf = tm.info()
    A, n_d0, n_cs = inf["anchors_per_row_tile"], inf["n_depth0_key_tiles"], inf["n_chain_sub_tiles"]
    M = orc.element_mask(L, K)
    for R in range(inf["n_row_tiles"]):
        rows = np.concatenate([d * L + np.arange(R * A, R * A + A) for d in range(K)])
        for c in range(n_d0):
            blk = M[np.ix_(rows, np.arange(64 * c, min(64 * c + 64, L)))]
            want = 0 if not blk.any() else (1 if blk.all() else 2)
            assert cls[R, c] == want
        for R2 in range(inf["n_row_tiles"]):
            for s in range(n_cs):
                ck = np.arange(64 * s, min(64 * s + 64, A * (K - 1)))
                cols = (1 + ck // A) * L + R2 * A + ck % A
                blk = M[np.ix_(rows, cols)]
                want = 0 if not blk.any() else (1 if blk.all() else 2)
                assert cls[R, n_d0 + R2 * n_cs + s] == want


def test_build_errors():
    lib = pe.load_library()
    out = C.c_void_p()
    i32p = C.POINTER(C.c_int32)

    def build(L, K, b, S, dev=-1, outp=C.byref(out)):
        arr = None if b is None else (C.c_int32 * len(b))(*b)
        return lib.peagle_build_tilemap(L, K, arr, S, dev, outp)

    assert build(128, 4, None, 1, -1, None) == -2            # ENULL
    assert build(0, 4, None, 1) == -1                        # EINVAL
    assert build(128, 0, None, 1) == -1
    assert build(128, 200, None, 1) == -5                    # K > 128
    assert build(128, 4, None, 2) == -2                      # bounds missing
    assert build(128, 4, [0, 64, 100], 2) == -4              # does not end at L_max
    assert build(128, 4, [0, 64, 64, 128], 3) == -4          # not strictly increasing
    assert build(128, 4, [0, 40, 128], 2) == -4              # inner bound not a multiple of A = 32
    assert build(128, 4, [0, 64, 128], 2) == 0
    lib.peagle_tilemap_destroy(out)
    for code in range(0, -10, -1):
        assert len(pe.peagle_strerror(code)) > 0


def test_compute_entry_points_validate_before_launch():
    """Every error path of the compute calls is reachable without a GPU (host-only tile map)."""
    lib = pe.load_library()
    tm = pe.peagle_build_tilemap(256, 8, [0, 128, 256], device=-1)
    one = C.c_void_p(16)  # never dereferenced: validation fails first

    def fwd(shape, seg=-1, q=one):
        return lib.peagle_attn_fwd(tm.handle, shape.c(), seg, q, one, one, one, one, None)

    ok = pe.Shape(256, 8, 4, 2, 64)
    assert fwd(pe.Shape(256, 8, 4, 3, 64)) == -1             # Hq % Hkv
    assert fwd(pe.Shape(256, 8, 4, 2, 96)) == -5             # head_dim
    assert fwd(pe.Shape(300, 8, 4, 2, 64)) == -3             # L > L_max
    assert fwd(pe.Shape(256, 4, 4, 2, 64)) == -3             # K mismatch
    assert fwd(pe.Shape(256, 8, 4, 2, 64, scale=-1.0)) == -1
    assert fwd(pe.Shape(256, 8, 4, 2, 64, layout=1)) == -5
    assert fwd(ok, q=None) == -2
    assert fwd(ok, seg=2) == -1
    assert fwd(ok) == -8                                     # host-only map cannot launch
    assert pe.peagle_workspace_bytes(tm, ok) > 256 * 8 * 4 * 4
    assert pe.peagle_workspace_bytes(tm, pe.Shape(256, 8, 4, 2, 96)) == 0
    rc = lib.peagle_attn_bwd(tm.handle, ok.c(), -1, one, one, one, one, one, one, one, one, one, 0, one, 16, None)
    assert rc == -6                                          # workspace too small
    rc = lib.peagle_attn_bwd(tm.handle, ok.c(), -1, one, one, one, one, one, one, one, one, one, 2, one, 1 << 40, None)
    assert rc == -1                                          # accumulate flag
    rc = lib.peagle_attn_step_partitioned(tm.handle, ok.c(), 1, 0, one, one, one, one, one, one, one, one, one, None,
                                          None, one, 1 << 40, None)
    assert rc == -1                                          # seg range
    rc = lib.peagle_attn_step_partitioned(tm.handle, ok.c(), 0, 2, one, one, one, one, one, one, one, one, one, None,
                                          None, None, 0, None)
    assert rc == -6


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_NAME", "libdoes_not_exist.so")
    monkeypatch.delenv("PEAGLE_ATTN_LIB", raising=False)
    with pytest.raises(ImportError):
        binding.load_library()


def test_trace_length_quantiles_hit_the_published_points():
    """The benchmark's length sweep passes through the three quantiles the paper prints (Fig. 1 caption)."""
    import bench
    assert bench.trace_lengths([0.5, 0.9, 0.99]) == [3904, 10816, 20000]   # 3,891 / 10,800 / 20,000 rounded up to 16
    ls = bench.trace_lengths([0.1, 0.25, 0.5, 0.75, 0.9, 0.95, 0.99])
    assert ls == sorted(ls) and all(l % 16 == 0 for l in ls)


# ----------------------------------------------------------------------------- sampled tile maps (host)

def _expand_all(tm, L):
    T = tm.tokens(L)
    bits = tm.expand_rows(L, -1, 0, T)
    return np.unpackbits(bits, axis=1, bitorder="little")[:, :T].astype(bool)


def _paper_example_counts():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "partition_example.txt")) as f:
        for line in f:
            tok = line.split("#")[0].split()
            if tok and tok[0] != "assign":
                vals[tok[0]] = [int(x) for x in tok[1:]]
    count = np.ones(vals["n"][0], dtype=np.int32)
    for g in range(1, vals["K"][0]):
        for p in vals[f"depth{g}"]:
            count[p - g] = g + 1
    return count, vals["K"][0]


@pytest.mark.parametrize("L,K,r,seed,bounds", [
    (16, 4, None, 0, None), (16, 4, None, 0, [0, 8, 16]), (300, 8, 0.8, 2, None), (300, 8, 0.8, 2, [0, 77, 150, 300]),
    (50, 3, 0.0, 3, None), (64, 5, 1.0, 4, None), (200, 16, 0.9, 5, [0, 100, 200]), (130, 1, 0.5, 6, None),
    (40, 128, 0.97, 7, None), (700, 4, 0.5, 8, [0, 1, 699, 700])])
def test_sampled_tilemap_expands_to_the_oracle_mask_bit_exactly(L, K, r, seed, bounds):
    from oracle import peagle_oracle as orc
    from peagle_inputs import cod_depth_counts
    if r is None:
        count, K = _paper_example_counts()
    else:
        count = cod_depth_counts(L, K, r, seed)
    tm = pe.peagle_build_tilemap_sampled(count, K, bounds, device=-1)
    ta, td = orc.cod_tokens(count)
    T = len(ta)
    inf = tm.info()
    assert inf["sampled"] == 1 and inf["tokens"] == T == tm.tokens(L)
    ref = orc.element_mask(L, K, tokens=(ta, td))
    assert np.array_equal(_expand_all(tm, L), ref)
    if bounds is not None:
        # per segment: exactly the rows of the segment's anchors, each with its full key set
        seen = np.zeros(T, dtype=int)
        for s in range(len(bounds) - 1):
            bits = np.unpackbits(tm.expand_rows(L, s, 0, T), axis=1, bitorder="little")[:, :T].astype(bool)
            rows = (ta >= bounds[s]) & (ta < bounds[s + 1])
            assert np.array_equal(bits[rows], ref[rows]) and not bits[~rows].any()
            seen += rows
        assert (seen == 1).all()
    # every row tile is packed: no tile could take the next anchor, and none crosses a segment boundary
    assert inf["n_row_tiles"] >= -(-T // 128)
    with pytest.raises(pe.PeagleError):
        tm.tokens(L - 1) if L > 1 else tm.tokens(L + 1)


def test_sampled_tilemap_packs_rows_densely():
    from peagle_inputs import cod_depth_counts
    L, K = 4096, 8
    count = cod_depth_counts(L, K, 0.8, 2)
    tm = pe.peagle_build_tilemap_sampled(count, K, [0, 1024, 2048, 3072, 4096], device=-1)
    inf = tm.info()
    T = int(count.sum())
    assert inf["tokens"] == T
    # greedy packing leaves at most K-1 free rows per tile (plus one short tile per segment)
    assert inf["n_row_tiles"] <= -(-T // (128 - (K - 1))) + 4
    dense = pe.peagle_build_tilemap(L, K, [0, 1024, 2048, 3072, 4096], device=-1).info()
    assert inf["n_row_tiles"] < 0.6 * dense["n_row_tiles"]


def test_sampled_tilemap_build_rejects_bad_arguments():
    lib = pe.load_library()
    import ctypes as C
    out = C.c_void_p()
    good = (C.c_int32 * 4)(1, 2, 3, 1)
    assert lib.peagle_build_tilemap_sampled(None, 4, 3, None, 1, 0, -1, C.byref(out)) == -2
    assert lib.peagle_build_tilemap_sampled(good, 4, 3, None, 1, 0, -1, None) == -2
    assert lib.peagle_build_tilemap_sampled(good, 0, 3, None, 1, 0, -1, C.byref(out)) == -1
    assert lib.peagle_build_tilemap_sampled(good, 4, 2, None, 1, 0, -1, C.byref(out)) == -1          # a count above K
    assert lib.peagle_build_tilemap_sampled((C.c_int32 * 4)(1, 0, 1, 1), 4, 3, None, 1, 0, -1, C.byref(out)) == -1
    assert lib.peagle_build_tilemap_sampled(good, 4, 129, None, 1, 0, -1, C.byref(out)) == -5
    assert lib.peagle_build_tilemap_sampled(good, 4, 3, (C.c_int32 * 3)(0, 3, 5), 2, 0, -1, C.byref(out)) == -4
    assert lib.peagle_build_tilemap_sampled(good, 4, 3, None, 2, 0, -1, C.byref(out)) == -2
    assert lib.peagle_build_tilemap_sampled(good, 4, 3, None, 1, 2, -1, C.byref(out)) == -1          # unknown assignment
    assert out.value is None
    assert lib.peagle_tilemap_tokens(None, 4) == -1


def test_sampled_map_serves_only_its_own_length():
    """Compute entry points reject another L for a sampled map on the host (no GPU involved)."""
    import ctypes as C
    lib = pe.load_library()
    tm = pe.peagle_build_tilemap_sampled([1, 2, 3, 4] * 16, 4, None, device=-1)
    one = C.c_void_p(16)   # never dereferenced: validation fails first

    def call(shape, ws=one, ws_bytes=1 << 40):
        return lib.peagle_attn_step_partitioned(tm.handle, shape.c(), 0, 1, one, one, one, one, one, one, one, one, one,
                                                None, None, ws, ws_bytes, None)
    assert call(pe.Shape(32, 4, 2, 1, 64)) == -3
    assert call(pe.Shape(64, 4, 2, 1, 64), ws=None) == -6
    assert call(pe.Shape(64, 4, 2, 1, 64)) == -8                                    # host-only map cannot launch
    assert pe.peagle_workspace_bytes(tm, pe.Shape(64, 4, 2, 1, 64)) > 0
    assert pe.peagle_workspace_bytes(tm, pe.Shape(32, 4, 2, 1, 64)) == 0


@pytest.mark.parametrize("L,K,r,seed,S", [(16, 4, None, 0, 2), (16, 4, None, 0, 3), (300, 8, 0.8, 2, 4), (257, 8, 1.0, 3, 3),
                                           (90, 3, 0.6, 4, 5), (40, 16, 0.9, 5, 2), (64, 1, 1.0, 6, 4)])
def test_algorithm1_assignment_matches_the_oracle_partition(L, K, r, seed, S):
    """With PEAGLE_ASSIGN_ALGORITHM1 the rows each segment computes are exactly the positions Algorithm 1
    assigns to it (oracle partition_assign, boundaries B_s = s n / S), and every row carries its full
    key set; the by-anchor assignment differs only in where the chains of the boundary anchors go."""
    from oracle import peagle_oracle as orc
    from peagle_inputs import cod_depth_counts
    if r is None:
        count, K = _paper_example_counts()
    else:
        count = cod_depth_counts(L, K, r, seed)
    ta, td = orc.cod_tokens(count)
    T = len(ta)
    positions = [sorted((ta[td == g] + g).tolist()) for g in range(int(td.max()) + 1)]
    A, N = orc.partition_assign(positions, S, L)
    want = np.array([A[d][a + d] for a, d in zip(ta.tolist(), td.tolist())])
    bounds = [-(-s * L // S) for s in range(S + 1)]                  # p in segment s  <=>  ceil(s n/S) <= p < ceil((s+1) n/S)
    tm = pe.peagle_build_tilemap_sampled(count, K, bounds, device=-1, assignment=pe.ASSIGN_ALGORITHM1)
    ref = orc.element_mask(L, K, tokens=(ta, td))
    for s in range(S):
        bits = np.unpackbits(tm.expand_rows(L, s, 0, T), axis=1, bitorder="little")[:, :T].astype(bool)
        rows = want == s
        assert np.array_equal(bits.any(axis=1), rows), s           # every row sees itself, so a computed row is non-empty
        assert np.array_equal(bits[rows], ref[rows])
        # the keys a segment touches: its own positions plus the cumulative depth-0 context N_s
        touched = np.nonzero(bits.any(axis=0))[0]
        allowed = set(np.nonzero(rows)[0].tolist()) | set(N[s])       # depth-0 token index == position
        assert set(touched.tolist()) <= allowed
    assert np.array_equal(_expand_all(tm, L), ref)
    if r is None and S == 2:
        # the printed dependency: position 8 at depth 2 shares the segment of position 7 at depth 1 (segment 0)
        tok = {(int(a), int(d)): t for t, (a, d) in enumerate(zip(ta, td))}
        bits0 = np.unpackbits(tm.expand_rows(L, 0, 0, T), axis=1, bitorder="little")[:, :T].astype(bool)
        assert bits0[tok[(6, 2)]].any() and bits0[tok[(6, 1)]].any()  # anchor 6: positions 7 (depth 1) and 8 (depth 2)


# ----------------------------------------------------------------------------- packed batches (host)

@pytest.mark.parametrize("seq_lens,K,r,seed,bounds,assign", [
    ((16,), 4, None, 0, None, 0),
    ((5, 3, 8), 3, None, 1, None, 0),
    ((100, 37, 64, 1, 90), 8, None, 2, None, 0),
    ((100, 37, 64, 1, 90), 8, None, 2, [0, 100, 137, 201, 202, 292], 0),        # one segment per sequence
    ((100, 37, 64, 1, 90), 8, 0.8, 3, [0, 50, 120, 292], 0),                      # segments cut across sequences
    ((100, 37, 64, 1, 90), 8, 0.8, 3, [0, 50, 120, 292], 1),
    ((70, 70, 70), 4, 0.5, 4, [0, 64, 128, 210], 1),
    ((130,) * 3, 1, None, 5, [0, 200, 390], 0),
    ((3, 2), 128, 0.95, 6, None, 0),
])
def test_packed_tilemap_expands_to_the_oracle_mask_bit_exactly(seq_lens, K, r, seed, bounds, assign):
    from oracle import peagle_oracle as orc
    from peagle_inputs import cod_depth_counts
    L = sum(seq_lens)
    count = None if r is None else cod_depth_counts(L, K, r, seed)
    tm = pe.peagle_build_tilemap_packed(seq_lens, K, count, bounds, device=-1, assignment=assign)
    tok = orc.packed_tokens(seq_lens, K, count)
    T = len(tok[0])
    assert tm.tokens(L) == T
    ref = orc.element_mask(L, K, tokens=tok)
    assert np.array_equal(_expand_all(tm, L), ref)
    if bounds is not None:
        seen = np.zeros(T, dtype=int)
        for s in range(len(bounds) - 1):
            bits = np.unpackbits(tm.expand_rows(L, s, 0, T), axis=1, bitorder="little")[:, :T].astype(bool)
            rows = bits.any(axis=1)
            assert np.array_equal(bits[rows], ref[rows])
            seen += rows
        assert (seen == 1).all()                                    # every row is computed in exactly one segment


def test_packed_dense_single_sequence_equals_the_dense_map():
    """One sequence, nothing dropped: the general builder must describe the same mask as the
    position-invariant dense map (tile geometry may differ; the expansion may not)."""
    L, K = 200, 8
    a = pe.peagle_build_tilemap_packed((L,), K, None, None, device=-1)
    b = pe.peagle_build_tilemap(L, K, None, device=-1)
    assert np.array_equal(_expand_all(a, L), _expand_all(b, L))
    assert a.info()["n_row_tiles"] == b.info()["n_row_tiles"]       # 16 anchors x 8 depths per tile either way


def test_packed_build_rejects_bad_arguments():
    lib = pe.load_library()
    out = C.c_void_p()
    i32 = C.c_int32
    assert lib.peagle_build_tilemap_packed(None, 8, 2, (i32 * 3)(0, 5, 9), 2, None, 1, 0, -1, C.byref(out)) == -4   # ends before L
    assert lib.peagle_build_tilemap_packed(None, 8, 2, (i32 * 3)(0, 5, 5), 2, None, 1, 0, -1, C.byref(out)) == -4   # empty sequence
    assert lib.peagle_build_tilemap_packed(None, 8, 2, None, 2, None, 1, 0, -1, C.byref(out)) == -2
    assert lib.peagle_build_tilemap_packed(None, 8, 2, (i32 * 3)(0, 5, 8), 0, None, 1, 0, -1, C.byref(out)) == -1
    assert out.value is None


# ----------------------------------------------------------------------------- rebuilding a map in place (host)

def test_rebuild_in_place_gives_the_same_map_as_a_fresh_build():
    from oracle import peagle_oracle as orc
    from peagle_inputs import cod_depth_counts
    K = 8
    tm = pe.peagle_build_tilemap_sampled(cod_depth_counts(300, K, 0.8, 1), K, [0, 100, 300], device=-1)
    cases = [((500,), 0.8, 2, [0, 250, 500], 0), ((40,), 0.5, 3, None, 1), ((100, 37, 64), 0.9, 4, [0, 90, 201], 1),
             ((300,), None, 5, None, 0)]
    for seq_lens, r, seed, bounds, assign in cases:
        L = sum(seq_lens)
        count = None if r is None else cod_depth_counts(L, K, r, seed)
        tm.rebuild(seq_lens, count, bounds, assign)
        fresh = pe.peagle_build_tilemap_packed(seq_lens, K, count, bounds, device=-1, assignment=assign)
        a, b = tm.info(), fresh.info()
        assert {k: a[k] for k in a if k != "device_bytes"} == {k: b[k] for k in b if k != "device_bytes"}
        tok = orc.packed_tokens(seq_lens, K, count)
        assert np.array_equal(_expand_all(tm, L), orc.element_mask(L, K, tokens=tok))
        S = 1 if bounds is None else len(bounds) - 1
        T = tm.tokens(L)
        for s in range(S):
            assert np.array_equal(tm.expand_rows(L, s, 0, T), fresh.expand_rows(L, s, 0, T))


def test_rebuild_rejects_bad_arguments_and_keeps_the_map():
    from peagle_inputs import cod_depth_counts
    lib = pe.load_library()
    K, L = 4, 64
    count = cod_depth_counts(L, K, 0.7, 9)
    tm = pe.peagle_build_tilemap_sampled(count, K, None, device=-1)
    before = _expand_all(tm, L)
    i32 = C.c_int32
    bad = (i32 * L)(*([5] * L))                                          # counts above K
    assert lib.peagle_tilemap_rebuild(tm.handle, bad, L, None, 1, None, 1, 0, None) == -1
    assert lib.peagle_tilemap_rebuild(tm.handle, None, L, None, 2, None, 1, 0, None) == -2
    assert lib.peagle_tilemap_rebuild(tm.handle, None, L, None, 1, (i32 * 3)(0, 70, 64), 2, 0, None) == -4
    assert lib.peagle_tilemap_rebuild(None, None, L, None, 1, None, 1, 0, None) == -2
    assert np.array_equal(_expand_all(tm, L), before)
    dense = pe.peagle_build_tilemap(L, K, None, device=-1)
    assert lib.peagle_tilemap_rebuild(dense.handle, None, L, None, 1, None, 1, 0, None) == -5


def test_random_position_sets_expand_to_the_oracle_mask():
    """Seeded sweep over batches, depths, retention rates, segmentations and both assignments: the general
    builder against the oracle's element mask, bit for bit, and every row in exactly one segment."""
    from oracle import peagle_oracle as orc
    from peagle_inputs import cod_depth_counts
    rng = np.random.default_rng(2024)
    for case in range(40):
        K = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 33]))
        n_seq = int(rng.integers(1, 5))
        seq_lens = tuple(int(x) for x in rng.integers(1, 150, size=n_seq))
        L = sum(seq_lens)
        r = float(rng.choice([0.0, 0.3, 0.6, 0.8, 0.95, 1.0]))
        count = None if rng.random() < 0.25 else cod_depth_counts(L, K, r, int(rng.integers(1 << 30)))
        S = int(rng.integers(1, 5))
        bounds = None
        if S > 1 and L > S:
            cuts = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False))
            bounds = [0] + [int(c) for c in cuts] + [L]
        assign = int(rng.integers(0, 2))
        what = f"case {case}: seq_lens={seq_lens} K={K} r={r} sampled={count is not None} bounds={bounds} assign={assign}"
        tm = pe.peagle_build_tilemap_packed(seq_lens, K, count, bounds, device=-1, assignment=assign)
        tok = orc.packed_tokens(seq_lens, K, count)
        T = len(tok[0])
        ref = orc.element_mask(L, K, tokens=tok)
        assert tm.tokens(L) == T, what
        assert np.array_equal(_expand_all(tm, L), ref), what
        if bounds is not None:
            seen = np.zeros(T, dtype=int)
            for s in range(len(bounds) - 1):
                bits = np.unpackbits(tm.expand_rows(L, s, 0, T), axis=1, bitorder="little")[:, :T].astype(bool)
                rows = bits.any(axis=1)
                assert np.array_equal(bits[rows], ref[rows]), what
                seen += rows
            assert (seen == 1).all(), what
        cls = tm.classes()
        inf = tm.info()
        assert (cls == 1).sum() == inf["n_full"] and (cls == 2).sum() == inf["n_partial"], what


# ----------------------------------------------------------------------------- rotary embedding: host side

def test_rope_position_ids_equal_the_oracle_for_every_kind_of_map():
    """Position p = anchor + depth (Sec. 3), restarting per sequence of a packed batch: index work, bit-exact."""
    from peagle_inputs import cod_depth_counts
    tm = pe.peagle_build_tilemap(300, 5, None, device=-1)
    for L in (300, 129, 1):
        np.testing.assert_array_equal(pe.peagle_rope_position_ids(tm, L), orc.position_ids(L, 5))
        assert pe.peagle_rope_positions(tm, L) == L + 4
    count = cod_depth_counts(200, 8, 0.7, 3)
    tm = pe.peagle_build_tilemap_sampled(count, 8, [0, 90, 200], device=-1)
    want = orc.position_ids(200, 8, tokens=orc.cod_tokens(count))
    np.testing.assert_array_equal(pe.peagle_rope_position_ids(tm, 200), want)
    assert pe.peagle_rope_positions(tm, 200) == want.max() + 1
    seq_lens = (100, 37, 64, 1, 90)
    count = cod_depth_counts(sum(seq_lens), 8, 0.8, 4)
    tm = pe.peagle_build_tilemap_packed(seq_lens, 8, count, None, device=-1)
    want = orc.position_ids(sum(seq_lens), 8, tokens=orc.packed_tokens(seq_lens, 8, count))
    np.testing.assert_array_equal(pe.peagle_rope_position_ids(tm, sum(seq_lens)), want)
    assert pe.peagle_rope_positions(tm, sum(seq_lens)) == want.max() + 1
    # a rebuild replaces the position ids with the map
    tm.rebuild((50, 242), cod_depth_counts(292, 8, 0.6, 5))
    want = orc.position_ids(292, 8, tokens=orc.packed_tokens((50, 242), 8, cod_depth_counts(292, 8, 0.6, 5)))
    np.testing.assert_array_equal(pe.peagle_rope_position_ids(tm, 292), want)


def test_rope_entry_points_validate_before_launch():
    lib = pe.load_library()
    tm = pe.peagle_build_tilemap(256, 8, [0, 128, 256], device=-1)
    one = C.c_void_p(16)  # never dereferenced: validation fails first
    ok = pe.Shape(256, 8, 4, 2, 64)
    assert lib.peagle_rope_table(C.c_float(500000.0), 64, 10, None, None) == -2
    assert lib.peagle_rope_table(C.c_float(1.0), 64, 10, one, None) == -1           # base must exceed 1
    assert lib.peagle_rope_table(C.c_float(1e4), 64, 0, one, None) == -1
    assert lib.peagle_rope_table(C.c_float(1e4), 96, 10, one, None) == -5
    assert lib.peagle_rope_positions(tm.handle, 257) == -1
    assert lib.peagle_rope_rotate(tm.handle, ok.c(), one, 4, one, 262, 0, one, None) == -3   # table covers too few positions
    assert lib.peagle_rope_rotate(tm.handle, ok.c(), one, 4, None, 263, 0, one, None) == -2
    assert lib.peagle_rope_rotate(tm.handle, ok.c(), one, 0, one, 263, 0, one, None) == -1
    assert lib.peagle_rope_rotate(tm.handle, ok.c(), one, 4, one, 263, 2, one, None) == -1
    assert lib.peagle_rope_rotate(tm.handle, ok.c(), one, 4, one, 263, 0, one, None) == -8   # host-only map
    assert pe.peagle_rope_workspace_bytes(tm, ok) >= pe.peagle_workspace_bytes(tm, ok) + 256 * 8 * (4 + 2) * 64 * 2

    def step(table=one, n_pos=263, ws=1 << 40, seg=(0, 2)):
        return lib.peagle_attn_step_partitioned_rope(tm.handle, ok.c(), seg[0], seg[1], one, one, one, one, table, n_pos,
                                                     one, one, one, one, one, None, None, one, ws, None)
    assert step(table=None) == -2
    assert step(n_pos=262) == -3
    assert step(ws=pe.peagle_workspace_bytes(tm, ok)) == -6      # the plain workspace is too small
    assert step(seg=(2, 1)) == -1
    assert step() == -8


# ----------------------------------------------------------------------------- inference-side drafting: host side

def test_draft_decode_validates_before_launch():
    lib = pe.load_library()
    one = C.c_void_p(16)  # never dereferenced: validation fails first

    def call(shape, q=one, ws=one, ws_bytes=1 << 40):
        return lib.peagle_draft_decode(shape.c(), q, one, one, one, one, one, one, one, one, None, ws, ws_bytes, None)

    ok = pe.DecodeShape(4, 7, 64, 8, 64, 100, 20)
    assert call(pe.DecodeShape(0, 7, 64, 8, 64, 100, 20)) == -1
    assert call(pe.DecodeShape(4, 7, 64, 6, 64, 100, 20)) == -1          # Hq % Hkv
    assert call(pe.DecodeShape(4, 7, 64, 8, 96, 100, 20)) == -5          # head_dim
    assert call(pe.DecodeShape(4, 7, 64, 2, 64, 100, 20)) == -5          # K * group > 128 rows
    assert call(pe.DecodeShape(4, 7, 64, 8, 64, 100, 20, scale=0.0)) == -1
    assert call(pe.DecodeShape(4, 7, 64, 8, 64, 0, 20)) == -1
    assert call(pe.DecodeShape(4, 7, 64, 8, 64, 100, (1 << 24) + 1)) == -5     # context length would overflow
    assert call(pe.DecodeShape(70000, 7, 64, 8, 64, 100, 20)) == -5            # more requests than a grid dimension
    assert call(ok, q=None) == -2
    assert call(ok, ws=None) == -6
    assert call(ok, ws_bytes=pe.peagle_draft_decode_workspace_bytes(ok) - 1) == -6
    assert lib.peagle_draft_decode_workspace_bytes(pe.DecodeShape(4, 7, 64, 8, 96, 100, 20).c()) == 0
    assert pe.peagle_draft_decode_splits(pe.DecodeShape(4, 7, 64, 8, 96, 100, 20)) == -1
    # split count: at least four pages per piece, never more than 32 pieces, at least one
    assert pe.peagle_draft_decode_splits(ok) == 5
    assert pe.peagle_draft_decode_splits(pe.DecodeShape(1, 3, 8, 8, 64, 10, 1)) == 1
    assert pe.peagle_draft_decode_splits(pe.DecodeShape(2, 3, 8, 1, 64, 5000, 4000)) == 32
    assert pe.peagle_draft_decode_splits(pe.DecodeShape(512, 3, 8, 8, 64, 5000, 4000)) == 1


def test_draft_decode_static_validates_before_launch():
    """The entry point with the library's own scratch array: same checks, and shapes whose partial records
    exceed the array are refused with the workspace error."""
    lib = pe.load_library()
    one = C.c_void_p(16)  # never dereferenced: validation fails first

    def call(shape, q=one):
        return lib.peagle_draft_decode_static(shape.c(), q, one, one, one, one, one, one, one, one, None, None)

    assert call(pe.DecodeShape(0, 7, 64, 8, 64, 100, 20)) == -1
    assert call(pe.DecodeShape(4, 7, 64, 8, 96, 100, 20)) == -5
    assert call(pe.DecodeShape(4, 7, 64, 8, 64, 100, 20), q=None) == -2
    big = pe.DecodeShape(4096, 7, 64, 8, 64, 8, 1)
    assert pe.peagle_draft_decode_workspace_bytes(big) > 32 << 20
    assert call(big) == -6


def test_decode_input_generator_scatters_the_context_over_pages():
    from peagle_inputs import PAGE_TOKENS, make_decode_inputs
    inp = make_decode_inputs([0, 1, 64, 65, 200], K=3, Hq=4, Hkv=2, D=64, seed=9)
    assert PAGE_TOKENS == 64 and inp["max_pages"] == 4 and inp["n_pages"] == 0 + 1 + 1 + 2 + 4 + 3
    used = inp["block_table"][inp["block_table"] >= 0]
    assert len(set(used.tolist())) == len(used) == 8                     # every block has a page of its own
    for c, n in enumerate(inp["ctx_len"]):
        for t in range(int(n)):
            page = inp["block_table"][c, t // 64]
            assert np.array_equal(inp["k_pages"][page, :, t % 64], inp["k_ctx"][c][t])
            assert np.array_equal(inp["v_pages"][page, :, t % 64], inp["v_ctx"][c][t])


def test_rope_shared_entry_point_validates_before_launch():
    lib = pe.load_library()
    tm = pe.peagle_build_tilemap(256, 8, [0, 128, 256], device=-1)
    one = C.c_void_p(16)
    ok = pe.Shape(256, 8, 4, 2, 64)

    def call(k_shared=one, n_pos=263, ws=1 << 40):
        return lib.peagle_attn_step_rope_shared(tm.handle, ok.c(), one, one, k_shared, one, one, one, one, n_pos, one, one,
                                                one, one, one, one, one, one, ws, None)
    assert call(k_shared=None) == -2
    assert call(n_pos=262) == -3
    assert call(ws=pe.peagle_rope_workspace_bytes(tm, ok)) == -6       # the rotary workspace alone is too small
    assert call() == -8
    need = pe.peagle_rope_shared_workspace_bytes(tm, ok)
    # beside the rotary workspace: one fp32 row of Hkv x D per wave (4) of each of the 16 row tiles' chain-tile
    # workgroups, for dK and for dV - and no [T, Hkv, D] tensor of any kind (D = 64)
    assert need == pe.peagle_rope_workspace_bytes(tm, ok) + 2 * (16 * 4) * (2 * 64) * 4
