"""GPU parity tests of the rotary-embedding step (Sec. 2 of the paper: LLaMA 3 style drafter with
RoPE; position p = anchor + depth, Sec. 3): table, rotation kernel, and the attention step on
unrotated Q / K with gradients returned in the unrotated frame, against the fp64 oracle.
Tolerances as for the plain step: forward max-abs <= 1e-2 / rel-L2 <= 5e-3, gradients rel-L2 <= 1e-2."""
import numpy as np
import pytest
import torch

import paper_2602_01469_amd as pe
from gpu_harness import Run, SampledRun, attach_rope, bf16_to_f64, max_abs, rand_bits, rel_l2, to_dev_bf16
from oracle import peagle_oracle as orc
from peagle_inputs import CONFIGS, bf16_bits_to_f64, cod_depth_counts, f32_to_bf16_bits, make_inputs
from test_gpu_parity import (FWD_REL, GRAD_REL, LSE_ABS, PART_REL, _check_against_oracle, _check_o_abs)

pytestmark = pytest.mark.gpu
BASE = 500000.0      # LLaMA 3
# The attention reads the rotated Q and K from bf16 tensors (as it reads every Q and K), so against the
# fp64 oracle - which rotates the bf16 inputs without rounding again - every score carries the rounding of
# its 2D rotated operands: standard deviation scale * sqrt(2D) * 2^-9 / sqrt(3) = 1.6e-3 for unit-variance
# inputs at scale = 1/sqrt(D).  A row's LSE moves by at most its largest score error; five standard
# deviations on top of the plain path's bound (2^-8 from the bf16 probabilities):
LSE_ABS_ROPE = LSE_ABS + 8e-3
# The same score errors d_j move an output element by sum_j p_j (v_j - O) d_j, standard deviation
# 1.6e-3 * sqrt(sum_j p_j^2 (v_j - O)^2) <= 1.6e-3 for a row whose weight sits on a few keys of unit-variance V;
# five standard deviations on top of the plain path's bound.  Every case is also compared at the plain bound with
# the oracle fed the rotated operands as stored (bf16), which carries no such term.
O_ABS_ROPE_EXTRA = 8e-3


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


@pytest.mark.parametrize("D,n_pos,base", [(64, 4104, 500000.0), (128, 20488, 500000.0), (64, 300, 10000.0)])
def test_rope_table_matches_closed_form(D, n_pos, base):
    print(f"case rope table D={D} n_pos={n_pos} base={base}", flush=True)
    table = torch.empty((n_pos, 2, D // 2), dtype=torch.float32, device="cuda")
    pe.peagle_rope_table(base, D, n_pos, table)
    got = table.double().cpu().numpy()
    a = orc.rope_angles(np.arange(n_pos), D, base)
    # fp32 rounding of a value in [-1, 1] is at most 2^-25; the double-precision angle adds < 1e-11
    assert np.abs(got[:, 0] - np.cos(a)).max() <= 2.0 ** -24
    assert np.abs(got[:, 1] - np.sin(a)).max() <= 2.0 ** -24


def _maps():
    count = cod_depth_counts(300, 8, 0.7, 11)
    seq_lens = (100, 37, 64, 1, 90)
    pcount = cod_depth_counts(sum(seq_lens), 4, 0.8, 12)
    return [
        ("dense_cropped", lambda: pe.peagle_build_tilemap(256, 8, None, device=0), 219, 8, None),
        ("sampled", lambda: pe.peagle_build_tilemap_sampled(count, 8, None, device=0), 300, 8, orc.cod_tokens(count)),
        ("packed", lambda: pe.peagle_build_tilemap_packed(seq_lens, 4, pcount, None, device=0), sum(seq_lens), 4,
         orc.packed_tokens(seq_lens, 4, pcount)),
    ]


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("which", [0, 1, 2])
def test_rope_rotation_kernel_matches_oracle(which, D):
    name, build, L, K, tokens = _maps()[which]
    print(f"case rope rotate {name} D={D}", flush=True)
    tm = build()
    T = tm.tokens(L)
    H = 3
    xb = rand_bits((T, H, D), 700 + which)
    x = to_dev_bf16(xb)
    shape = pe.Shape(L, K, H, H, D)
    n_pos = pe.peagle_rope_positions(tm, L)
    table = torch.empty((n_pos, 2, D // 2), dtype=torch.float32, device="cuda")
    pe.peagle_rope_table(BASE, D, n_pos, table)
    pos = orc.position_ids(L, K, tokens)
    for inverse in (False, True):
        out = torch.full((T, H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        pe.peagle_rope_rotate(tm, shape, x, table, out, inverse=inverse)
        got = bf16_to_f64(out)
        ref = orc.rope_rotate(bf16_bits_to_f64(xb), pos, BASE, inverse=inverse)
        # one rounding to bf16 (half an ulp: 2^-9 relative) plus fp32 arithmetic on two products
        bound = np.abs(ref) * 2.0 ** -8 + 1e-6
        assert (np.abs(got - ref) <= bound).all(), (name, inverse, np.abs(got - ref).max())
        assert rel_l2(got, ref) <= 3e-3


ROPE_CASES = [
    # name, L, K, Hq, Hkv, D, seed, bounds, L_max
    ("one_tile", 16, 8, 4, 2, 64, 800, None, None),
    ("segments", 256, 8, 4, 2, 64, 810, [0, 64, 128, 256], None),
    ("segments_cropped", 219, 8, 4, 2, 64, 820, [0, 64, 128, 256], 256),
    ("d128_segments", 200, 4, 4, 2, 128, 830, [0, 96, 200], None),
    ("several_tiles_group_of_6", 700, 4, 6, 1, 64, 840, [0, 256, 512, 700], None),
    ("k1", 300, 1, 2, 2, 64, 850, None, None),
    ("odd_group_d128", 70, 8, 9, 3, 128, 860, None, None),
    ("k32_positions_far_past_the_anchors", 20, 32, 2, 1, 64, 870, None, None),
    ("k5_segments", 60, 5, 4, 2, 64, 880, [0, 25, 60], None),
]


def _oracle_rope(qb, kb, vb, dob, L, K, scale, bounds, tokens=None):
    q, k, v, do = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    return orc.attn_step_rope(q, k, v, do, L, K, scale, bounds if bounds is not None else [0, L], BASE, tokens=tokens)


def _round_bf16(x):
    return bf16_bits_to_f64(f32_to_bf16_bits(x.astype(np.float32)))


def _oracle_rope_stored(qb, kb, vb, dob, L, K, scale, bounds, tokens=None):
    """The oracle with the rotated Q and K rounded to their bf16 storage format before the attention, which
    removes the operand-rounding term above: the plain step's tolerances then apply unchanged."""
    q, k, v, do = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    pos = orc.position_ids(L, K, tokens)
    qr, kr = _round_bf16(orc.rope_rotate(q, pos, BASE)), _round_bf16(orc.rope_rotate(k, pos, BASE))
    if tokens is None:
        r = dict(orc.attn_step_partitioned(qr, kr, v, do, L, K, scale, bounds if bounds is not None else [0, L]))
    else:
        r = dict(orc.attn_backward(qr, kr, v, do, L, K, scale, tokens=tokens))
    r["dQ"] = orc.rope_rotate(r["dQ"], pos, BASE, inverse=True)
    r["dK"] = orc.rope_rotate(r["dK"], pos, BASE, inverse=True)
    return r


def _check_rope(got, qb, kb, vb, dob, L, K, scale, bounds, name, tokens=None):
    _check_against_oracle(got, _oracle_rope(qb, kb, vb, dob, L, K, scale, bounds, tokens), name, lse_abs=LSE_ABS_ROPE,
                          o_abs_extra=O_ABS_ROPE_EXTRA)
    _check_against_oracle(got, _oracle_rope_stored(qb, kb, vb, dob, L, K, scale, bounds, tokens), name + " (stored operands)")


@pytest.mark.parametrize("name,L,K,Hq,Hkv,D,seed,bounds,L_max", ROPE_CASES, ids=[c[0] for c in ROPE_CASES])
def test_rope_step_matches_oracle(name, L, K, Hq, Hkv, D, seed, bounds, L_max):
    print(f"case rope {name}: L={L} K={K} Hq={Hq} Hkv={Hkv} D={D} seed={seed} bounds={bounds} L_max={L_max}", flush=True)
    T = L * K
    qb, kb, vb, dob = (rand_bits((T, Hq, D), seed), rand_bits((T, Hkv, D), seed + 1), rand_bits((T, Hkv, D), seed + 2),
                       rand_bits((T, Hq, D), seed + 3))
    tm = pe.peagle_build_tilemap(L_max or L, K, bounds, device=0)
    S = 1 if bounds is None else len(bounds) - 1
    r = attach_rope(Run(tm, L, K, Hq, Hkv, D, qb, kb, vb, dob), BASE)
    r.step_rope(0, S)
    got = r.results()
    ob = None if bounds is None else [min(b, L) for b in bounds if b < L] + [L]
    _check_rope(got, qb, kb, vb, dob, L, K, r.shape.scale, ob, name)
    if S > 1:
        # a run resumed in the middle accumulates dK in the unrotated frame exactly as one call does
        r2 = attach_rope(Run(tm, L, K, Hq, Hkv, D, qb, kb, vb, dob), BASE)
        r2.step_rope(0, 1)
        r2.step_rope(1, S)
        g2 = r2.results()
        for n in got:
            assert np.array_equal(g2[n], got[n]), n
        # and one unpartitioned pass agrees to the accumulation-order tolerance
        tm1 = pe.peagle_build_tilemap(L_max or L, K, None, device=0)
        r3 = attach_rope(Run(tm1, L, K, Hq, Hkv, D, qb, kb, vb, dob), BASE)
        r3.step_rope(0, 1)
        g3 = r3.results()
        for n in ("O", "LSE", "dQ"):
            assert np.array_equal(g3[n], got[n]), n
        for n in ("dK", "dV"):
            assert rel_l2(g3[n], got[n]) <= PART_REL, n


def test_rope_step_equals_the_plain_step_on_rotated_inputs():
    """The step on unrotated inputs must be the plain step applied to the rotated copies the rotation
    kernel produces: O, LSE, dV bit-identical; dQ, dK the plain ones turned back (checked through the oracle's
    inverse rotation of the plain step's fp32 / bf16 outputs, to rounding)."""
    L, K, Hq, Hkv, D = 384, 8, 8, 2, 64
    print(f"case rope vs plain: L={L} K={K}", flush=True)
    T = L * K
    qb, kb, vb, dob = (rand_bits((T, Hq, D), 870), rand_bits((T, Hkv, D), 871), rand_bits((T, Hkv, D), 872),
                       rand_bits((T, Hq, D), 873))
    bounds = [0, 128, 384]
    tm = pe.peagle_build_tilemap(L, K, bounds, device=0)
    r = attach_rope(Run(tm, L, K, Hq, Hkv, D, qb, kb, vb, dob), BASE)
    r.step_rope(0, 2)
    got = r.results()
    q_rot = torch.empty_like(r.q)
    k_rot = torch.empty_like(r.k)
    pe.peagle_rope_rotate(tm, r.shape, r.q, r.rope_table, q_rot)
    pe.peagle_rope_rotate(tm, pe.Shape(L, K, Hkv, Hkv, D), r.k, r.rope_table, k_rot)
    p = Run(tm, L, K, Hq, Hkv, D, qb, kb, vb, dob)
    p.q, p.k = q_rot, k_rot
    p.step(0, 2)
    plain = p.results()
    for n in ("O", "LSE", "dV"):
        assert np.array_equal(plain[n], got[n]), n
    pos = orc.position_ids(L, K)
    dk_back = orc.rope_rotate(plain["dK"], pos, BASE, inverse=True)
    assert rel_l2(got["dK"], dk_back) <= 1e-6                 # fp32 sums turned back in fp32
    dq_back = orc.rope_rotate(plain["dQ"], pos, BASE, inverse=True)
    assert rel_l2(got["dQ"], dq_back) <= 6e-3                 # the plain dQ was rounded to bf16 before turning


ROPE_LISTED = [
    # name, seq_lens, K, Hq, Hkv, D, retention, seed, bounds, assignment
    ("sampled_alg1", (300,), 8, 4, 2, 64, 0.7, 900, [0, 100, 300], 1),
    ("sampled_d128", (200,), 4, 2, 1, 128, 0.8, 910, None, 0),
    ("packed_dense", (100, 37, 64, 1, 90), 8, 4, 2, 64, None, 920, None, 0),
    ("packed_sampled_segments", (150, 260, 90), 8, 4, 1, 64, 0.8, 930, [0, 150, 333, 500], 1),
]


@pytest.mark.parametrize("name,seq_lens,K,Hq,Hkv,D,ret,seed,bounds,assign", ROPE_LISTED, ids=[c[0] for c in ROPE_LISTED])
def test_rope_step_on_sampled_and_packed_maps(name, seq_lens, K, Hq, Hkv, D, ret, seed, bounds, assign):
    print(f"case rope {name}: seq_lens={seq_lens} K={K} Hq={Hq} Hkv={Hkv} D={D} r={ret} bounds={bounds}", flush=True)
    L = sum(seq_lens)
    count = None if ret is None else cod_depth_counts(L, K, ret, seed)
    tm = pe.peagle_build_tilemap_packed(seq_lens, K, count, bounds, device=0, assignment=assign)
    tokens = orc.packed_tokens(seq_lens, K, count)
    T = tm.tokens(L)
    assert T == len(tokens[0])
    qb, kb, vb, dob = (rand_bits((T, Hq, D), seed), rand_bits((T, Hkv, D), seed + 1), rand_bits((T, Hkv, D), seed + 2),
                       rand_bits((T, Hq, D), seed + 3))
    r = attach_rope(SampledRun(tm, L, K, Hq, Hkv, D, qb, kb, vb, dob), BASE)
    S = 1 if bounds is None else len(bounds) - 1
    r.step_rope(0, S)
    got = r.results()
    _check_rope(got, qb, kb, vb, dob, L, K, r.shape.scale, None, name, tokens=tokens)


def test_rope_full_size_c3_sampled_rows():
    """c3 in the launch configuration the benchmark's rotary run times: oracle on sampled rows of one KV group."""
    cfg = CONFIGS["c3_median"]
    print(f"case rope {cfg.name}: generating inputs", flush=True)
    qb, kb, vb, dob = make_inputs(cfg)
    b = cfg.seg_bounds()
    tm = pe.peagle_build_tilemap(cfg.L, cfg.K, b, device=0)
    r = attach_rope(Run(tm, cfg.L, cfg.K, cfg.Hq, cfg.Hkv, cfg.D, qb, kb, vb, dob, cfg.scale), BASE)
    print(f"case rope {cfg.name}: partitioned step, {len(b) - 1} segments", flush=True)
    r.step_rope(0, len(b) - 1)
    got = r.results()
    assert not any(np.isnan(got[n]).any() for n in got)
    print(f"case rope {cfg.name}: oracle on sampled rows", flush=True)
    L, K, g = cfg.L, cfg.K, cfg.Hkv - 1
    grp = cfg.Hq // cfg.Hkv
    hs = slice(g * grp, (g + 1) * grp)
    pos = orc.position_ids(L, K)
    q = orc.rope_rotate(bf16_bits_to_f64(qb[:, hs]), pos, BASE)
    k = orc.rope_rotate(bf16_bits_to_f64(kb[:, g:g + 1]), pos, BASE)
    v, do = bf16_bits_to_f64(vb[:, g:g + 1]), bf16_bits_to_f64(dob[:, hs])
    rng = np.random.default_rng(1)
    anchors = np.unique(np.concatenate([[0, 1, 63, 64, L // 2, L - 1], rng.integers(0, L, size=6)]))
    rows = np.concatenate([d * L + anchors for d in range(K)])
    ref = orc.attn_backward(q, k, v, do, L, K, cfg.scale, rows=rows, row_block=256)
    assert rel_l2(got["O"][rows][:, hs], ref["O"]) <= FWD_REL
    _check_o_abs(got["O"][rows][:, hs], ref["O"], "rope " + cfg.name, O_ABS_ROPE_EXTRA)
    assert max_abs(got["LSE"][hs][:, rows], ref["LSE"]) <= LSE_ABS_ROPE
    assert rel_l2(got["dQ"][rows][:, hs], orc.rope_rotate(ref["dQ"], pos[rows], BASE, inverse=True)) <= GRAD_REL
    tail = 40       # keys of the last anchors are seen only by rows of those anchors
    rows2 = np.concatenate([d * L + np.arange(L - tail, L) for d in range(K)])
    ref2 = orc.attn_backward(q, k, v, do, L, K, cfg.scale, rows=rows2, row_block=256)
    dk_ref = orc.rope_rotate(ref2["dK"][rows2], pos[rows2], BASE, inverse=True)
    assert rel_l2(got["dK"][rows2][:, g:g + 1], dk_ref) <= GRAD_REL
    assert rel_l2(got["dV"][rows2][:, g:g + 1], ref2["dV"][rows2]) <= GRAD_REL
    # softmax rows sum to one whatever the rotation: sum_keys dV = sum_rows dO per KV head
    dof = bf16_bits_to_f64(dob)
    rhs = dof.sum(axis=0).reshape(cfg.Hkv, grp, cfg.D).sum(axis=1)
    assert np.abs(got["dV"].sum(axis=0) - rhs).max() <= 2e-3 * np.abs(dof).sum(axis=0).reshape(cfg.Hkv, grp, cfg.D).sum(axis=1).max()


def test_rope_step_replays_from_a_hip_graph():
    """The rotary step records kernel launches only (two more than the plain step): three replays, with new
    inputs written and the program synchronising between them, each bit-identical to the eager result."""
    L, K, Hq, Hkv, D = 640, 8, 8, 2, 64
    bounds = [0, 256, 640]
    print(f"case rope graph replay: L={L} K={K} bounds={bounds}", flush=True)
    T = L * K
    tm = pe.peagle_build_tilemap(L, K, bounds, device=0)

    def bits(seed):
        return (rand_bits((T, Hq, D), seed), rand_bits((T, Hkv, D), seed + 1), rand_bits((T, Hkv, D), seed + 2),
                rand_bits((T, Hq, D), seed + 3))

    r = attach_rope(Run(tm, L, K, Hq, Hkv, D, *bits(2100)), BASE)
    r.step_rope(0, 2)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pe.peagle_attn_step_partitioned_rope(tm, r.shape, 0, 2, r.q, r.k, r.v, r.do, r.rope_table, r.o, r.lse, r.dq,
                                             r.dk, r.dv, None, None, r.ws, torch.cuda.current_stream())
    for rep in range(3):
        qb, kb, vb, dob = bits(2200 + 10 * rep)
        for dst, src in ((r.q, qb), (r.k, kb), (r.v, vb), (r.do, dob)):
            dst.copy_(to_dev_bf16(src))
        graph.replay()
        torch.cuda.synchronize()
        got = {n: t.clone() for n, t in (("o", r.o), ("lse", r.lse), ("dq", r.dq), ("dk", r.dk), ("dv", r.dv))}
        for t in (r.o, r.dq):
            t.fill_(float("nan"))
        r.step_rope(0, 2)
        torch.cuda.synchronize()
        for n, t in (("o", r.o), ("lse", r.lse), ("dq", r.dq), ("dk", r.dk), ("dv", r.dv)):
            assert torch.equal(got[n], t), (rep, n)
    ref = _oracle_rope(qb, kb, vb, dob, L, K, r.shape.scale, bounds)
    _check_against_oracle(r.results(), ref, "rope graph replay", lse_abs=LSE_ABS_ROPE, o_abs_extra=O_ABS_ROPE_EXTRA)


SHARED_CASES = [
    # name, seq_lens, K, Hq, Hkv, D, retention, seed, bounds, dense map?
    ("dense_segments", (256,), 8, 4, 2, 64, None, 3000, [0, 64, 128, 256], True),
    ("dense_d128", (200,), 4, 4, 2, 128, None, 3010, [0, 96, 200], True),
    ("dense_k1_no_chain", (300,), 1, 2, 2, 64, None, 3020, None, True),
    ("sampled", (300,), 8, 4, 2, 64, 0.7, 3030, [0, 100, 300], False),
    ("packed", (100, 37, 64, 1, 90), 8, 4, 1, 64, 0.8, 3040, None, False),
    ("dense_k2_one_chain_tile", (200,), 2, 4, 2, 64, None, 3050, [0, 64, 200], True),
    ("dense_k5", (120,), 5, 2, 1, 64, None, 3060, [0, 50, 120], True),
    ("dense_k32", (20,), 32, 2, 1, 64, None, 3070, None, True),
]


@pytest.mark.parametrize("name,seq_lens,K,Hq,Hkv,D,ret,seed,bounds,dense", SHARED_CASES, ids=[c[0] for c in SHARED_CASES])
def test_rope_step_with_shared_chain_vectors_matches_oracle(name, seq_lens, K, Hq, Hkv, D, ret, seed, bounds, dense):
    """First-layer form (Sec. 2): depth-0 keys / values of their own, one shared vector for every other position."""
    print(f"case rope shared {name}: seq_lens={seq_lens} K={K} Hq={Hq} Hkv={Hkv} D={D} r={ret} bounds={bounds}", flush=True)
    L = sum(seq_lens)
    if dense:
        tm = pe.peagle_build_tilemap(L, K, bounds, device=0)
        tokens = None
    else:
        count = None if ret is None else cod_depth_counts(L, K, ret, seed)
        tm = pe.peagle_build_tilemap_packed(seq_lens, K, count, bounds, device=0)
        tokens = orc.packed_tokens(seq_lens, K, count)
    T = tm.tokens(L)
    qb, dob = rand_bits((T, Hq, D), seed), rand_bits((T, Hq, D), seed + 1)
    k0b, v0b = rand_bits((L, Hkv, D), seed + 2), rand_bits((L, Hkv, D), seed + 3)
    ksb, vsb = rand_bits((Hkv, D), seed + 4), rand_bits((Hkv, D), seed + 5)
    shape = pe.Shape(L, K, Hq, Hkv, D)
    n_pos = pe.peagle_rope_positions(tm, L)
    table = torch.empty((n_pos, 2, D // 2), dtype=torch.float32, device="cuda")
    pe.peagle_rope_table(BASE, D, n_pos, table)
    dev = {n: to_dev_bf16(x) for n, x in (("q", qb), ("do", dob), ("k0", k0b), ("v0", v0b), ("ks", ksb), ("vs", vsb))}
    nan = float("nan")
    o = torch.full((T, Hq, D), nan, dtype=torch.bfloat16, device="cuda")
    dq = torch.full((T, Hq, D), nan, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((Hq, T), nan, dtype=torch.float32, device="cuda")
    dk0 = torch.full((L, Hkv, D), nan, dtype=torch.float32, device="cuda")
    dv0 = torch.full((L, Hkv, D), nan, dtype=torch.float32, device="cuda")
    dks = torch.full((Hkv, D), nan, dtype=torch.float32, device="cuda")
    dvs = torch.full((Hkv, D), nan, dtype=torch.float32, device="cuda")
    ws = torch.empty(pe.peagle_rope_shared_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
    for rep in range(2):        # the second call reuses the workspace: identical bits
        pe.peagle_attn_step_rope_shared(tm, shape, dev["q"], dev["k0"], dev["ks"], dev["v0"], dev["vs"], dev["do"], table, o,
                                        lse, dq, dk0, dv0, dks, dvs, ws)
        torch.cuda.synchronize()
        got = {"O": bf16_to_f64(o), "LSE": lse.double().cpu().numpy(), "dQ": bf16_to_f64(dq),
               "dK0": dk0.double().cpu().numpy(), "dV0": dv0.double().cpu().numpy(),
               "dK_shared": dks.double().cpu().numpy(), "dV_shared": dvs.double().cpu().numpy()}
        if rep == 0:
            first = got
    for n in got:
        assert np.array_equal(first[n], got[n]), n
    f = bf16_bits_to_f64
    ob = bounds if bounds is not None else [0, L]
    ref = orc.attn_step_rope_shared(f(qb), f(k0b), f(ksb), f(v0b), f(vsb), f(dob), L, K, shape.scale, ob, BASE,
                                    tokens=tokens)
    assert not any(np.isnan(got[n]).any() for n in got)
    assert rel_l2(got["O"], ref["O"]) <= FWD_REL
    _check_o_abs(got["O"], ref["O"], name, O_ABS_ROPE_EXTRA)
    assert max_abs(got["LSE"], ref["LSE"]) <= LSE_ABS_ROPE
    for n in ("dQ", "dK0", "dV0"):
        assert rel_l2(got[n], ref[n]) <= GRAD_REL, n
    if K > 1:
        for n in ("dK_shared", "dV_shared"):
            assert rel_l2(got[n], ref[n]) <= GRAD_REL, n
    else:
        assert not got["dK_shared"].any() and not got["dV_shared"].any()
