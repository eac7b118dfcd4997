"""Pins for the fp64 oracle: every check compares it with something other than itself
(closed forms, library routines, brute force from the paper's dependency rules,
finite differences, values printed in the paper)."""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import peagle_oracle as orc
from peagle_inputs import CONFIGS, bf16_bits_to_f64, f32_to_bf16_bits, make_inputs, useful_pairs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(L, K, Hq, Hkv, D, seed):
    rng = np.random.default_rng(seed)
    T = L * K
    return (rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hkv, D)),
            rng.standard_normal((T, Hkv, D)), rng.standard_normal((T, Hq, D)))


# ----------------------------------------------------------------------------- mask

def _mask_from_dependency_rules(L, K):
    """Mask rebuilt in *position* coordinates from the paper's rules, by brute force:
    (p, d) with p = i + d depends on (p-1, d-1) transitively down to depth 1, sees
    itself, and sees the depth-0 context available to its anchor (positions <= p - d)."""
    T = L * K
    M = np.zeros((T, T), dtype=bool)
    for i, d in itertools.product(range(L), range(K)):
        r = d * L + i
        p = i + d
        for q0 in range(0, p - d + 1):          # depth-0 positions q0 <= p-d, anchor == position
            M[r, q0] = True
        pp, dd = p, d
        while dd >= 1:                          # self, then (p-1,d-1), (p-2,d-2), ... down to depth 1
            anchor = pp - dd
            M[r, dd * L + anchor] = True
            pp, dd = pp - 1, dd - 1
    return M


@pytest.mark.parametrize("L,K", [(1, 1), (5, 1), (7, 3), (16, 4), (9, 8)])
def test_mask_matches_dependency_rules(L, K):
    assert np.array_equal(orc.element_mask(L, K), _mask_from_dependency_rules(L, K))


@pytest.mark.parametrize("L,K", [(7, 3), (16, 4), (33, 8)])
def test_mask_scalar_predicate_agrees(L, K):
    M = orc.element_mask(L, K)
    for r in range(L * K):
        i, d = orc.token_coords(r, L)
        for c in range(L * K):
            j, e = orc.token_coords(c, L)
            assert M[r, c] == orc.visible(i, d, j, e)


@pytest.mark.parametrize("L,K", [(16, 4), (128, 4), (50, 8), (64, 1)])
def test_mask_closed_form_counts(L, K):
    M = orc.element_mask(L, K)
    T = L * K
    i, d = orc.token_coords(np.arange(T), L)
    assert np.array_equal(M.sum(axis=1), i + 1 + d)               # row (i,d) sees i+1 causal + d chain keys
    assert M.sum() == useful_pairs(L, K)
    col = M.sum(axis=0)
    j, e = orc.token_coords(np.arange(T), L)
    expect = np.where(e == 0, K * (L - j), K - e)                  # depth-0 key j: K*(L-j) rows; chain key: K-e rows
    assert np.array_equal(col, expect)
    # depth rule: no key of a deeper depth is ever visible
    assert not M[(d[:, None] < e[None, :])].any()


def test_useful_pairs_values():
    assert useful_pairs(128, 4) == 33792
    assert useful_pairs(2048, 4) == 8404992
    assert useful_pairs(4096, 8) == 67239936


def test_mask_k1_is_causal():
    assert np.array_equal(orc.element_mask(37, 1), np.tril(np.ones((37, 37), dtype=bool)))


@pytest.mark.parametrize("L1,L2,K", [(5, 12, 3), (16, 40, 4), (8, 9, 8)])
def test_mask_crop_invariance(L1, L2, K):
    """Position invariance (Sec. 3.1): the mask of the shorter sequence is the longer one's
    restricted to anchors < L1, in (anchor, depth) coordinates."""
    M1 = orc.element_mask(L1, K)
    M2 = orc.element_mask(L2, K)
    idx = np.array([orc.token_index(i, d, L2) for d in range(K) for i in range(L1)])
    assert np.array_equal(M2[np.ix_(idx, idx)], M1)


# ----------------------------------------------------------------------------- forward

def _torch_sdpa(q, k, v, mask=None, causal=False, scale=None):
    """Library routine: torch SDPA on CPU in fp64. q [T,H,D] -> [T,H,D]."""
    tq = torch.from_numpy(q).permute(1, 0, 2).unsqueeze(0)
    tk = torch.from_numpy(k).permute(1, 0, 2).unsqueeze(0)
    tv = torch.from_numpy(v).permute(1, 0, 2).unsqueeze(0)
    m = None if mask is None else torch.from_numpy(mask)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=m, is_causal=causal, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def test_depth0_rows_are_plain_causal_attention():
    L, K, Hq, Hkv, D = 48, 4, 4, 2, 16
    q, k, v, _ = _rand(L, K, Hq, Hkv, D, 3)
    scale = 0.37
    O, LSE = orc.attn_forward(q, k, v, L, K, scale)
    rep = Hq // Hkv
    ref = _torch_sdpa(q[:L], np.repeat(k[:L], rep, axis=1), np.repeat(v[:L], rep, axis=1), causal=True, scale=scale)
    assert np.allclose(O[:L], ref, rtol=1e-12, atol=1e-12)
    # LSE of depth-0 rows against scipy's logsumexp
    from scipy.special import logsumexp
    for h in range(Hq):
        g = h // rep
        S = scale * q[:L, h] @ k[:L, g].T
        S[np.triu_indices(L, 1)] = -np.inf
        assert np.allclose(LSE[h, :L], logsumexp(S, axis=1), rtol=1e-12, atol=1e-12)


def test_k1_whole_problem_is_causal_attention_fwd_bwd():
    L, K, Hq, Hkv, D = 40, 1, 2, 1, 8
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 4)
    scale = 1.0 / np.sqrt(D)
    r = orc.attn_backward(q, k, v, do, L, K, scale)
    tq = torch.from_numpy(q).requires_grad_()
    tk = torch.from_numpy(k).requires_grad_()
    tv = torch.from_numpy(v).requires_grad_()
    o = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], tk.permute(1, 0, 2).repeat_interleave(2, 0)[None],
        tv.permute(1, 0, 2).repeat_interleave(2, 0)[None], is_causal=True, scale=scale)[0].permute(1, 0, 2)
    (o * torch.from_numpy(do)).sum().backward()
    assert np.allclose(r["O"], o.detach().numpy(), atol=1e-12)
    assert np.allclose(r["dQ"], tq.grad.numpy(), atol=1e-12)
    assert np.allclose(r["dK"], tk.grad.numpy(), atol=1e-12)
    assert np.allclose(r["dV"], tv.grad.numpy(), atol=1e-12)


@pytest.mark.parametrize("L,K,Hq,Hkv,D", [(12, 3, 4, 2, 8), (16, 4, 4, 1, 16), (6, 8, 2, 2, 4)])
def test_library_autograd_with_independent_mask(L, K, Hq, Hkv, D):
    """Forward and all three gradients against torch autograd through its own SDPA, with the mask
    rebuilt from the dependency rules (not the oracle's builder) and GQA done by repeat_interleave."""
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 5)
    scale = 0.21
    r = orc.attn_backward(q, k, v, do, L, K, scale)
    M = torch.from_numpy(_mask_from_dependency_rules(L, K))
    rep = Hq // Hkv
    tq = torch.from_numpy(q).requires_grad_()
    tk = torch.from_numpy(k).requires_grad_()
    tv = torch.from_numpy(v).requires_grad_()
    o = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], tk.permute(1, 0, 2).repeat_interleave(rep, 0)[None],
        tv.permute(1, 0, 2).repeat_interleave(rep, 0)[None], attn_mask=M, scale=scale)[0].permute(1, 0, 2)
    (o * torch.from_numpy(do)).sum().backward()
    assert np.allclose(r["O"], o.detach().numpy(), atol=1e-12)
    assert np.allclose(r["dQ"], tq.grad.numpy(), atol=1e-11)
    assert np.allclose(r["dK"], tk.grad.numpy(), atol=1e-11)
    assert np.allclose(r["dV"], tv.grad.numpy(), atol=1e-11)


def test_softmax_rows_sum_to_one_and_lse_consistent():
    L, K, Hq, Hkv, D = 20, 4, 2, 1, 8
    q, k, v, _ = _rand(L, K, Hq, Hkv, D, 6)
    O, LSE, P = orc.attn_forward(q, k, v, L, K, 0.5, return_probs=True)
    assert np.allclose(P.sum(axis=2), 1.0, atol=1e-14)
    M = _mask_from_dependency_rules(L, K)
    assert (P[:, ~M] == 0).all()
    # P == exp(S - LSE) on visible entries
    S = 0.5 * np.einsum("rhd,chd->hrc", q, np.repeat(k, 2, axis=1))
    assert np.allclose(P[:, M], np.exp(S - LSE[:, :, None])[:, M], atol=1e-13)


def test_zero_query_closed_form():
    """Q == 0: uniform softmax, so O(i,d) is the mean of the visible V rows and LSE = ln(i+1+d)."""
    L, K, Hq, Hkv, D = 24, 4, 2, 2, 8
    _, k, v, do = _rand(L, K, Hq, Hkv, D, 7)
    q = np.zeros((L * K, Hq, D))
    r = orc.attn_backward(q, k, v, do, L, K, 0.3)
    for i, d in itertools.product(range(L), range(K)):
        t = d * L + i
        cnt = i + 1 + d
        for h in range(Hq):
            mean = (v[:i + 1, h].sum(axis=0) + sum(v[e * L + i, h] for e in range(1, d + 1))) / cnt
            assert np.allclose(r["O"][t, h], mean, atol=1e-13)
            assert np.isclose(r["LSE"][h, t], np.log(cnt), atol=1e-13)
    # dV closed form: each row spreads dO/count over its visible keys
    dV = np.zeros_like(v)
    for i, d in itertools.product(range(L), range(K)):
        t = d * L + i
        cnt = i + 1 + d
        for h in range(Hq):
            dV[:i + 1, h] += do[t, h] / cnt
            for e in range(1, d + 1):
                dV[e * L + i, h] += do[t, h] / cnt
    assert np.allclose(r["dV"], dV, atol=1e-12)


def test_constant_v_gives_constant_output():
    L, K, Hq, Hkv, D = 10, 3, 2, 1, 4
    q, k, _, _ = _rand(L, K, Hq, Hkv, D, 8)
    v = np.tile(np.arange(D, dtype=np.float64), (L * K, Hkv, 1))
    O, _ = orc.attn_forward(q, k, v, L, K, 1.0)
    assert np.allclose(O, np.arange(D), atol=1e-13)


# ----------------------------------------------------------------------------- backward

def test_finite_differences():
    L, K, Hq, Hkv, D = 6, 3, 4, 2, 4
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 9)
    scale = 0.45
    r = orc.attn_backward(q, k, v, do, L, K, scale)

    def loss(q_, k_, v_):
        O, _ = orc.attn_forward(q_, k_, v_, L, K, scale)
        return (O * do).sum()

    eps = 1e-6
    rng = np.random.default_rng(0)
    for name, arr, grad in (("q", q, r["dQ"]), ("k", k, r["dK"]), ("v", v, r["dV"])):
        flat = arr.reshape(-1)
        for idx in rng.choice(flat.size, size=40, replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            fp = loss(q, k, v)
            flat[idx] = old - eps
            fm = loss(q, k, v)
            flat[idx] = old
            fd = (fp - fm) / (2 * eps)
            assert np.isclose(fd, grad.reshape(-1)[idx], rtol=1e-6, atol=1e-8), (name, idx)


def test_backward_identities():
    L, K, Hq, Hkv, D = 14, 4, 2, 1, 8
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 10)
    scale = 0.3
    r = orc.attn_backward(q, k, v, do, L, K, scale)
    # sum_rows dQ . q == sum dK . k (both equal sum dS*S/scale*scale): the score gradient seen from both sides
    assert np.isclose((r["dQ"] * q).sum(), (r["dK"] * k).sum(), rtol=1e-12)
    # sum over keys of dV equals sum over rows of dO per KV head (softmax rows sum to 1)
    assert np.allclose(r["dV"].sum(axis=0)[0], do.sum(axis=(0, 1)), atol=1e-12)


# ----------------------------------------------------------------------------- partition

@pytest.mark.parametrize("bounds", [[0, 16], [0, 8, 16], [0, 4, 8, 12, 16], [0, 5, 16]])
def test_partitioned_equals_unpartitioned(bounds):
    L, K, Hq, Hkv, D = 16, 4, 4, 2, 8
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 11)
    full = orc.attn_backward(q, k, v, do, L, K, 0.35)
    part = orc.attn_step_partitioned(q, k, v, do, L, K, 0.35, bounds)
    for name in ("O", "LSE", "dQ", "dK", "dV"):
        assert np.allclose(full[name], part[name], atol=1e-13), name


def test_segment_rows_partition_all_rows_and_keys_cover_mask():
    L, K = 24, 4
    bounds = [0, 8, 16, 24]
    seen = []
    M = _mask_from_dependency_rules(L, K)
    for s in range(3):
        rows = orc.segment_rows(L, K, bounds[s], bounds[s + 1])
        cols = set(orc.segment_keys(L, K, bounds[s], bounds[s + 1]).tolist())
        seen.extend(rows.tolist())
        needed = set(np.nonzero(M[rows].any(axis=0))[0].tolist())
        assert needed <= cols                      # every key a row may see is present in its segment
    assert sorted(seen) == list(range(L * K))      # disjoint cover of all query rows


def _read_partition_example():
    d = {}
    assigns = []
    with open(os.path.join(GOLDEN, "partition_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "assign":
                assigns.append((int(tok[1][-1]), int(tok[2]), int(tok[3])))
            elif tok[0].startswith("depth"):
                d[tok[0]] = [int(x) for x in tok[1:]]
            else:
                d[tok[0]] = int(tok[1])
    return d, assigns


def test_partition_worked_example_from_paper():
    d, assigns = _read_partition_example()
    pos = [d[f"depth{g}"] for g in range(d["K"])]
    assert sum(len(p) for p in pos) == d["total"]
    A, N = orc.partition_assign(pos, d["S"], d["n"])
    for g, p, s in assigns:
        assert A[g][p] == s
    # every position shares the segment of its dependency (p-1, g-1) for g >= 2
    for g in range(2, d["K"]):
        for p in pos[g]:
            assert A[g][p] == A[g - 1][p - 1]
    assert N[0] == list(range(8)) and N[1] == list(range(16))
    assert all(A[0][p] == (0 if p < 8 else 1) for p in pos[0])


def test_cod_count_formula_value_from_paper():
    vals = {}
    with open(os.path.join(GOLDEN, "cod_count.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                a, b = line.split()
                vals[a] = float(b)
    got = orc.cod_position_count(int(vals["n"]), int(vals["K"]), vals["r"])
    assert abs(got - vals["approx"]) / vals["approx"] < vals["rel_tol"]
    assert abs(got - 34088.0) < 1.0
    assert orc.cod_position_count(16, 4, 1.0) == 64


# ----------------------------------------------------------------------------- input generator

def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(100000).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = bf16_bits_to_f64(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy())


def test_make_inputs_shapes_and_determinism():
    cfg = CONFIGS["c1_tiny"]
    a = make_inputs(cfg)
    b = make_inputs(cfg)
    assert a[0].shape == (512, 4, 64) and a[1].shape == (512, 1, 64) and a[3].shape == (512, 4, 64)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert a[0].dtype == np.uint16
    x = bf16_bits_to_f64(a[0])
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02


# ----------------------------------------------------------------------------- drop-token sampled sequences

def _paper_example_depth_counts():
    """Per-anchor depth counts of the worked example of Sec. 3.2 (positions at depth g minus g = anchors)."""
    d, _ = _read_partition_example()
    count = np.ones(d["n"], dtype=int)
    for g in range(1, d["K"]):
        for p in d[f"depth{g}"]:
            assert count[p - g] == g          # the predecessor (p-1, g-1) is kept: sets are nested per anchor
            count[p - g] = g + 1
    return count, d


def test_sampled_tokens_of_paper_example():
    count, d = _paper_example_depth_counts()
    ta, td = orc.cod_tokens(count)
    assert len(ta) == d["total"] == 38
    for g in range(d["K"]):
        assert sorted((ta[td == g] + g).tolist()) == d[f"depth{g}"]     # storage order: depth-major, positions ascending


def _sampled_mask_brute_force(count, K):
    """Mask over stored tokens rebuilt from the dependency rules in position coordinates."""
    ta, td = orc.cod_tokens(count)
    pos = {(int(a) + int(g), int(g)): t for t, (a, g) in enumerate(zip(ta, td))}   # (position, depth) -> token
    T = len(ta)
    M = np.zeros((T, T), dtype=bool)
    for (p, g), r in pos.items():
        for q0 in range(0, p - g + 1):
            M[r, pos[(q0, 0)]] = True
        pp, gg = p, g
        while gg >= 1:
            M[r, pos[(pp, gg)]] = True       # exists by nestedness
            pp, gg = pp - 1, gg - 1
    return M


def test_sampled_mask_matches_dependency_rules_and_is_a_submask_of_the_dense_one():
    count, d = _paper_example_depth_counts()
    K, L = d["K"], d["n"]
    ta, td = orc.cod_tokens(count)
    M = orc.element_mask(L, K, tokens=(ta, td))
    assert np.array_equal(M, _sampled_mask_brute_force(count, K))
    dense = orc.element_mask(L, K)
    idx = td * L + ta                                                   # same (anchor, depth) in the dense layout
    assert np.array_equal(M, dense[np.ix_(idx, idx)])
    assert np.array_equal(M.sum(axis=1), ta + 1 + td)                   # visible count is unchanged by sampling
    from peagle_inputs import useful_pairs_sampled
    assert M.sum() == useful_pairs_sampled(count)
    assert useful_pairs_sampled(np.full(L, K)) == useful_pairs(L, K)


def test_sampled_attention_equals_dense_attention_on_kept_rows():
    """Dropping positions removes rows and the keys only those rows could see, so a kept row's output
    equals the dense problem's output for the same (anchor, depth)."""
    count, d = _paper_example_depth_counts()
    K, L, Hq, Hkv, D = d["K"], d["n"], 2, 1, 8
    ta, td = orc.cod_tokens(count)
    qd, kd, vd, dod = _rand(L, K, Hq, Hkv, D, 21)
    idx = td * L + ta
    O, LSE = orc.attn_forward(qd[idx], kd[idx], vd[idx], L, K, 0.4, tokens=(ta, td))
    Od, LSEd = orc.attn_forward(qd, kd, vd, L, K, 0.4)
    assert np.allclose(O, Od[idx], atol=1e-13) and np.allclose(LSE, LSEd[:, idx], atol=1e-13)
    # gradients against torch autograd with the brute-force mask
    r = orc.attn_backward(qd[idx], kd[idx], vd[idx], dod[idx], L, K, 0.4, tokens=(ta, td))
    M = torch.from_numpy(_sampled_mask_brute_force(count, K))
    tq = torch.from_numpy(qd[idx]).requires_grad_()
    tk = torch.from_numpy(kd[idx]).requires_grad_()
    tv = torch.from_numpy(vd[idx]).requires_grad_()
    o = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], tk.permute(1, 0, 2).repeat_interleave(2, 0)[None],
        tv.permute(1, 0, 2).repeat_interleave(2, 0)[None], attn_mask=M, scale=0.4)[0].permute(1, 0, 2)
    (o * torch.from_numpy(dod[idx])).sum().backward()
    for name, t in (("dQ", tq), ("dK", tk), ("dV", tv)):
        assert np.allclose(r[name], t.grad.numpy(), atol=1e-11), name


def test_sampled_partition_by_algorithm_1_equals_single_pass():
    count, d = _paper_example_depth_counts()
    K, L, Hq, Hkv, D = d["K"], d["n"], 2, 1, 8
    ta, td = orc.cod_tokens(count)
    rng = np.random.default_rng(22)
    T = len(ta)
    q, k, v, do = (rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hkv, D)), rng.standard_normal((T, Hkv, D)),
                   rng.standard_normal((T, Hq, D)))
    full = orc.attn_backward(q, k, v, do, L, K, 0.3, tokens=(ta, td))
    for S in (2, 4):
        part = orc.attn_step_partitioned_sampled(q, k, v, do, count, K, 0.3, S)
        for name in ("O", "LSE", "dQ", "dK", "dV"):
            assert np.allclose(full[name], part[name], atol=1e-13), (S, name)


def test_cod_depth_counts_follow_geometric_retention():
    from peagle_inputs import cod_depth_counts
    L, K, r = 8192, 8, 0.8
    c = cod_depth_counts(L, K, r, seed=5)
    assert c.min() >= 1 and c.max() <= K
    sizes = [(c > g).sum() for g in range(K)]
    assert sizes[0] == L
    for g in range(1, K):
        assert sizes[g] == round(r * sizes[g - 1])
    assert abs(sum(sizes) - orc.cod_position_count(L, K, r)) < K          # the paper's n(1-r^K)/(1-r), up to rounding


# ----------------------------------------------------------------------------- packed batches

def _packed_mask_brute_force(seq_lens, K):
    """Block-diagonal assembly of the per-sequence masks (each rebuilt from the dependency rules) in the
    packed storage order t = d * L_total + global anchor."""
    Lt = sum(seq_lens)
    M = np.zeros((Lt * K, Lt * K), dtype=bool)
    base = 0
    for L in seq_lens:
        m = _mask_from_dependency_rules(L, K)
        idx = np.array([d * Lt + base + i for d in range(K) for i in range(L)])      # local t = d*L + i
        M[np.ix_(idx, idx)] = m
        base += L
    return M


@pytest.mark.parametrize("seq_lens,K", [((5, 3, 8), 3), ((1, 1, 1), 4), ((16,), 4), ((7, 20), 8)])
def test_packed_mask_is_block_diagonal(seq_lens, K):
    tok = orc.packed_tokens(seq_lens, K)
    Lt = sum(seq_lens)
    assert np.array_equal(orc.element_mask(Lt, K, tokens=tok), _packed_mask_brute_force(seq_lens, K))


def test_packed_attention_equals_each_sequence_alone():
    seq_lens, K, Hq, Hkv, D = (6, 11, 4), 4, 4, 2, 8
    Lt = sum(seq_lens)
    q, k, v, do = _rand(Lt, K, Hq, Hkv, D, 31)
    tok = orc.packed_tokens(seq_lens, K)
    r = orc.attn_backward(q, k, v, do, Lt, K, 0.3, tokens=tok)
    base = 0
    for L in seq_lens:
        idx = np.array([d * Lt + base + i for d in range(K) for i in range(L)])
        one = orc.attn_backward(q[idx], k[idx], v[idx], do[idx], L, K, 0.3)
        for n in ("O", "dQ", "dK", "dV"):
            assert np.allclose(r[n][idx], one[n], atol=1e-13), n
        assert np.allclose(r["LSE"][:, idx], one["LSE"], atol=1e-13)
        base += L
    # and against library autograd with the brute-force block mask
    M = torch.from_numpy(_packed_mask_brute_force(seq_lens, K))
    tq = torch.from_numpy(q).requires_grad_()
    tk = torch.from_numpy(k).requires_grad_()
    tv = torch.from_numpy(v).requires_grad_()
    o = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], tk.permute(1, 0, 2).repeat_interleave(2, 0)[None],
        tv.permute(1, 0, 2).repeat_interleave(2, 0)[None], attn_mask=M, scale=0.3)[0].permute(1, 0, 2)
    (o * torch.from_numpy(do)).sum().backward()
    assert np.allclose(r["O"], o.detach().numpy(), atol=1e-12)
    for name, t in (("dQ", tq), ("dK", tk), ("dV", tv)):
        assert np.allclose(r[name], t.grad.numpy(), atol=1e-11), name


def test_packed_sampled_tokens_keep_per_sequence_structure():
    from peagle_inputs import cod_depth_counts
    seq_lens, K = (9, 14, 5), 4
    Lt = sum(seq_lens)
    count = cod_depth_counts(Lt, K, 0.7, 3)
    ta, td, ts = orc.packed_tokens(seq_lens, K, count)
    M = orc.element_mask(Lt, K, tokens=(ta, td, ts))
    dense = _packed_mask_brute_force(seq_lens, K)
    idx = td * Lt + ta
    assert np.array_equal(M, dense[np.ix_(idx, idx)])
    start = np.concatenate([[0], np.cumsum(seq_lens)])[ts]
    assert np.array_equal(M.sum(axis=1), ta - start + 1 + td)


# ----------------------------------------------------------------------------- rotary embedding (Sec. 2)

def test_rope_two_dimensional_case_is_complex_multiplication():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 3, 2))
    pos = np.array([0, 1, 2, 5, 9, 100, 4097])
    got = orc.rope_rotate(x, pos, base=10000.0)
    z = (x[..., 0] + 1j * x[..., 1]) * np.exp(1j * pos.astype(np.float64))[:, None]   # D = 2: the only frequency is 1
    np.testing.assert_allclose(got[..., 0], z.real, rtol=0, atol=1e-12)
    np.testing.assert_allclose(got[..., 1], z.imag, rtol=0, atol=1e-12)


def test_rope_hand_computed_vector_and_frequencies():
    # D = 4, base 10000: frequencies 1 and 1/100; features (0,2) and (1,3) are the rotated pairs
    np.testing.assert_allclose(orc.rope_angles(np.array([3]), 4, 10000.0), [[3.0, 0.03]], rtol=1e-15)
    x = np.array([[[1.0, 0.0, 0.0, 2.0]]])
    got = orc.rope_rotate(x, np.array([3]), 10000.0)[0, 0]
    want = [np.cos(3.0), -2.0 * np.sin(0.03), np.sin(3.0), 2.0 * np.cos(0.03)]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)
    # LLaMA 3 base, D = 64: the slowest frequency is base^(-62/64)
    a = orc.rope_angles(np.array([1]), 64, 500000.0)
    assert abs(a[0, 31] - 500000.0 ** (-62.0 / 64.0)) < 1e-18 and a[0, 0] == 1.0


def test_rope_is_an_isometry_with_the_transpose_as_inverse():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((40, 2, 16))
    y = rng.standard_normal((40, 2, 16))
    pos = rng.integers(0, 30000, size=40)
    rx = orc.rope_rotate(x, pos, 500000.0)
    np.testing.assert_allclose(np.linalg.norm(rx, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    np.testing.assert_allclose(orc.rope_rotate(rx, pos, 500000.0, inverse=True), x, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(orc.rope_rotate(x, np.zeros(40, dtype=int), 500000.0), x)
    # <R x, y> = <x, R^T y>: the inverse is the transpose (what the gradient takes)
    lhs = (rx * y).sum()
    rhs = (x * orc.rope_rotate(y, pos, 500000.0, inverse=True)).sum()
    assert abs(lhs - rhs) < 1e-10
    # scores depend on the position difference only
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    s1 = (orc.rope_rotate(q, np.array([17]), 1e4) * orc.rope_rotate(k, np.array([5]), 1e4)).sum()
    s2 = (orc.rope_rotate(q, np.array([1012]), 1e4) * orc.rope_rotate(k, np.array([1000]), 1e4)).sum()
    assert abs(s1 - s2) < 1e-10


def test_position_ids_follow_the_rows_named_in_the_paper_example():
    # Sec. 3.2 names rows by (position, depth); in its worked dependency example the row (position 8, depth 2)
    # hangs on the row (position 7, depth 1): both belong to anchor 6, and the stored tokens carry those positions.
    count, d = _paper_example_depth_counts()
    ta, td = orc.cod_tokens(count)
    pos = orc.position_ids(len(count), d["K"], tokens=(ta, td))
    for g in range(d["K"]):
        assert sorted(pos[td == g].tolist()) == d[f"depth{g}"]
    t8 = [t for t in range(len(ta)) if td[t] == 2 and pos[t] == 8][0]
    t7 = [t for t in range(len(ta)) if td[t] == 1 and pos[t] == 7][0]
    assert ta[t8] == ta[t7] == 6
    # dense layout t = d*L + i
    L, K = 5, 3
    np.testing.assert_array_equal(orc.position_ids(L, K), [0, 1, 2, 3, 4, 1, 2, 3, 4, 5, 2, 3, 4, 5, 6])
    # packed batch: positions restart with every sequence
    tok = orc.packed_tokens([3, 2], 2)
    np.testing.assert_array_equal(orc.position_ids(5, 2, tokens=tok), [0, 1, 2, 0, 1, 1, 2, 3, 1, 2])


def test_rope_step_is_invariant_under_a_common_position_shift():
    L, K, Hq, Hkv, D = 12, 3, 4, 2, 8
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 31)
    pos = orc.position_ids(L, K)
    a = orc.attn_step_rope(q, k, v, do, L, K, 0.3, [0, 5, 12], 10000.0)
    b = orc.attn_step_rope(q, k, v, do, L, K, 0.3, [0, 5, 12], 10000.0, pos=pos + 777)
    for name in ("O", "LSE", "dV", "dQ", "dK"):       # raw-space gradients are shift invariant too
        np.testing.assert_allclose(a[name], b[name], rtol=0, atol=1e-9)
    # with every token at one position all rotations are equal: scores, and with them every output
    # and raw-space gradient, are those of the unrotated step
    same = orc.attn_step_rope(q, k, v, do, L, K, 0.3, [0, 5, 12], 10000.0, pos=np.full(L * K, 9))
    plain = orc.attn_step_partitioned(q, k, v, do, L, K, 0.3, [0, 5, 12])
    for name in ("O", "LSE", "dV"):
        np.testing.assert_allclose(same[name], plain[name], rtol=0, atol=1e-9)
    np.testing.assert_allclose(same["dQ"], plain["dQ"], rtol=0, atol=1e-9)
    np.testing.assert_allclose(same["dK"], plain["dK"], rtol=0, atol=1e-9)


def test_rope_step_gradients_against_finite_differences():
    L, K, Hq, Hkv, D = 6, 3, 2, 1, 4
    q, k, v, do = _rand(L, K, Hq, Hkv, D, 33)
    base, scale, bounds = 100.0, 0.4, [0, 2, 6]
    r = orc.attn_step_rope(q, k, v, do, L, K, scale, bounds, base)

    def loss(qq, kk):
        pos = orc.position_ids(L, K)
        O, _ = orc.attn_forward(orc.rope_rotate(qq, pos, base), orc.rope_rotate(kk, pos, base), v, L, K, scale)
        return float((O * do).sum())

    eps = 1e-6
    rng = np.random.default_rng(34)
    for _ in range(12):
        t, d = int(rng.integers(L * K)), int(rng.integers(D))
        h = int(rng.integers(Hq))
        e = np.zeros_like(q)
        e[t, h, d] = eps
        fd = (loss(q + e, k) - loss(q - e, k)) / (2 * eps)
        assert abs(fd - r["dQ"][t, h, d]) < 1e-7 * max(1.0, abs(fd))
        e = np.zeros_like(k)
        e[t, 0, d] = eps
        fd = (loss(q, k + e) - loss(q, k - e)) / (2 * eps)
        assert abs(fd - r["dK"][t, 0, d]) < 1e-7 * max(1.0, abs(fd))


def test_rope_step_on_a_packed_batch_equals_each_sequence_alone():
    K, Hq, Hkv, D = 3, 2, 1, 8
    seq_lens = [5, 7]
    tok = orc.packed_tokens(seq_lens, K)
    L = sum(seq_lens)
    rng = np.random.default_rng(35)
    T = len(tok[0])
    q, k, v, do = (rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hkv, D)),
                   rng.standard_normal((T, Hkv, D)), rng.standard_normal((T, Hq, D)))
    both = orc.attn_step_rope(q, k, v, do, L, K, 0.35, [0, L], 500000.0, tokens=tok)
    for s, n in enumerate(seq_lens):
        sel = np.nonzero(tok[2] == s)[0]           # depth-major inside the sequence as well
        one = orc.attn_step_rope(q[sel], k[sel], v[sel], do[sel], n, K, 0.35, [0, n], 500000.0)
        for name in ("O", "dQ", "dK", "dV"):
            np.testing.assert_allclose(both[name][sel], one[name], rtol=0, atol=1e-10)


# ----------------------------------------------------------------------------- inference-side drafting (Sec. 2)

def test_draft_decode_equals_the_last_anchor_of_the_training_problem():
    """The K rows of a drafting step are the rows (n, 0..K-1) of the expanded training sequence of n+1
    anchors: same visible keys (mask rebuilt from the dependency rules), same outputs."""
    n, K, Hq, Hkv, D = 9, 4, 4, 2, 8
    L = n + 1
    q, k, v, _ = _rand(L, K, Hq, Hkv, D, 41)
    M = _mask_from_dependency_rules(L, K)
    rows = np.array([d * L + n for d in range(K)])
    O, LSE = orc.draft_decode(q[rows], k[rows], v[rows], k[:n], v[:n], 0.3)
    for d in range(K):                                   # visible set of row (n, d): context, (n,0), own chain
        vis = set(np.nonzero(M[rows[d]])[0].tolist())
        assert vis == set(range(n)) | {e * L + n for e in range(d + 1)}
    Ot, LSEt = orc.attn_forward(q, k, v, L, K, 0.3, rows=rows)
    np.testing.assert_allclose(O, Ot, rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, LSEt, rtol=0, atol=1e-12)


def test_draft_decode_against_library_attention_and_closed_forms():
    n, K, Hq, Hkv, D = 37, 5, 6, 2, 16
    rng = np.random.default_rng(42)
    qn, kn, vn = rng.standard_normal((K, Hq, D)), rng.standard_normal((K, Hkv, D)), rng.standard_normal((K, Hkv, D))
    kc, vc = rng.standard_normal((n, Hkv, D)), rng.standard_normal((n, Hkv, D))
    O, LSE = orc.draft_decode(qn, kn, vn, kc, vc, 0.25)
    mask = torch.ones(K, n + K, dtype=torch.bool)
    mask[:, n:] = torch.tril(torch.ones(K, K, dtype=torch.bool))       # new key e visible to row d iff e <= d
    keys = torch.from_numpy(np.concatenate([kc, kn])).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    vals = torch.from_numpy(np.concatenate([vc, vn])).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(qn).permute(1, 0, 2), keys, vals,
                                                           attn_mask=mask, scale=0.25)
    np.testing.assert_allclose(O, ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)
    # zero queries: uniform weights over the n + d + 1 visible keys
    O0, LSE0 = orc.draft_decode(np.zeros_like(qn), kn, vn, kc, vc, 0.25)
    allv = np.concatenate([vc, vn])
    for d in range(K):
        np.testing.assert_allclose(O0[d, 0], allv[:n + d + 1, 0].mean(axis=0), rtol=0, atol=1e-12)
        np.testing.assert_allclose(LSE0[:, d], np.log(n + d + 1), rtol=0, atol=1e-12)
    # empty context: row 0 sees only the new depth-0 key
    O1, LSE1 = orc.draft_decode(qn, kn, vn, kc[:0], vc[:0], 0.25)
    np.testing.assert_allclose(O1[0, 0], vn[0, 0], rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE1[0, 0], 0.25 * qn[0, 0] @ kn[0, 0], rtol=0, atol=1e-12)


def test_shared_chain_vectors_gradients_against_finite_differences():
    """First-layer form (Sec. 2): one key / value vector for all multi-token positions.  Gradients with
    respect to those vectors by central differences of the loss through the plain forward."""
    L, K, Hq, Hkv, D = 5, 3, 2, 1, 4
    rng = np.random.default_rng(51)
    T = L * K
    q, do = rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hq, D))
    k0, v0 = rng.standard_normal((L, Hkv, D)), rng.standard_normal((L, Hkv, D))
    ks, vs = rng.standard_normal((Hkv, D)), rng.standard_normal((Hkv, D))
    base, scale = 50.0, 0.45
    r = orc.attn_step_rope_shared(q, k0, ks, v0, vs, do, L, K, scale, [0, 2, 5], base)

    def loss(k0_, ks_, v0_, vs_):
        pos = orc.position_ids(L, K)
        k = np.concatenate([k0_] + [ks_[None]] * (T - L))
        v = np.concatenate([v0_] + [vs_[None]] * (T - L))
        O, _ = orc.attn_forward(orc.rope_rotate(q, pos, base), orc.rope_rotate(k, pos, base), v, L, K, scale)
        return float((O * do).sum())

    eps = 1e-6
    for d in range(D):
        e = np.zeros_like(ks)
        e[0, d] = eps
        fd = (loss(k0, ks + e, v0, vs) - loss(k0, ks - e, v0, vs)) / (2 * eps)
        assert abs(fd - r["dK_shared"][0, d]) < 1e-7 * max(1.0, abs(fd))
        fd = (loss(k0, ks, v0, vs + e) - loss(k0, ks, v0, vs - e)) / (2 * eps)
        assert abs(fd - r["dV_shared"][0, d]) < 1e-7 * max(1.0, abs(fd))
        e0 = np.zeros_like(k0)
        e0[3, 0, d] = eps
        fd = (loss(k0 + e0, ks, v0, vs) - loss(k0 - e0, ks, v0, vs)) / (2 * eps)
        assert abs(fd - r["dK0"][3, 0, d]) < 1e-7 * max(1.0, abs(fd))
        fd = (loss(k0, ks, v0 + e0, vs) - loss(k0, ks, v0 - e0, vs)) / (2 * eps)
        assert abs(fd - r["dV0"][3, 0, d]) < 1e-7 * max(1.0, abs(fd))
    # K = 1: there is no multi-token position, so the shared vectors receive no gradient
    r1 = orc.attn_step_rope_shared(q[:L], k0, ks, v0, vs, do[:L], L, 1, scale, [0, L], base)
    assert np.array_equal(r1["dK_shared"], np.zeros((Hkv, D))) and np.array_equal(r1["dV_shared"], np.zeros((Hkv, D)))
