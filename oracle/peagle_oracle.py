"""fp64 CPU oracle for the parallel-drafting attention of the P-EAGLE drafter.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it is
used by ``tests/``, the smoke check and the ``cpu_baseline`` leg of the benchmark.  It
shares no code with the HIP path and never reads a value produced by it.

What is computed (paper, Sec. 3): a sequence of ``L`` tokens is expanded to ``T = L*K``
positions, one per (anchor ``i``, prediction depth ``d``); depth ``d`` predicts the
token ``d+1`` ahead.  Attention over the expanded sequence runs under the
parallel-prediction mask (Sec. 3, second paragraph, and Sec. 3.2 "Challenge 2"):

  * a row of depth ``d`` sees depths ``<= d`` only;
  * in position coordinates ``p = i + d`` the row ``(p, d)`` depends on ``(p-1, d-1)``,
    hence on the whole chain down to depth 1, i.e. in anchor coordinates on
    ``(i, 1), ..., (i, d)`` (self included);
  * depth-0 keys are the ordinary causal context: anchors ``j <= i``.

Readings of points the paper leaves open are listed in the design notes of this
repository; the ones that matter here: a row attends to itself and to ``(i, 0)``;
no other anchor's keys at depth >= 1 are visible; the expanded sequence is stored
depth-major, ``t = d*L + i``; query head ``h`` uses KV head ``h // (Hq/Hkv)`` (the
drafter is a LLaMA-3 style decoder, Sec. 2); the log-sum-exp is natural-log and
includes the softmax scale.

Conditional Drop-token sampling (the PARD paragraph of Sec. 3; position-count formula of
Sec. 3.2) keeps only some positions at depths >= 1.  Because a kept position p at depth g needs
p-1 at depth g-1 (Sec. 3.2, Challenge 2), the kept set is, per anchor, a prefix of its depths:
anchor i keeps depths 0..n_i-1.  Every function below therefore also accepts an explicit token
list ``tokens = (anchor[t], depth[t])`` in storage order; the mask is the same predicate
evaluated on those coordinates.

Everything is plain dense fp64: an explicit boolean mask evaluated element by element
from the predicate, ``numpy`` matmuls, max-subtracted softmax.  The only blocking is
over query rows, to bound memory; there is no tiling, fusion or reordering.

Pins (tests/test_oracle_pins.py): closed-form visible counts, causal reduction at
depth 0 and at K=1 against an independent library routine, library autograd with an
independently built mask, zero-query closed forms, finite differences, crop
invariance, and the worked partition example of Sec. 3.2 / Fig. 4 for the segment
assignment routine.  The sampled-sequence path is pinned on that same worked example (its 38
positions): token list against the printed position sets, mask against a brute-force rebuild
from the dependency rules and against the dense mask restricted to kept positions, outputs
against the dense problem's kept rows, gradients against library autograd, and Algorithm 1
partitioning against the single pass.  Packed batches: mask against the block-diagonal assembly of
per-sequence masks rebuilt from the dependency rules, outputs against each sequence alone and
against library autograd.  Rotary embedding (Sec. 2): the D = 2 case against complex multiplication,
a hand-computed D = 4 vector, norm and inverse identities, position ids against the rows the worked
example of Sec. 3.2 names by (position, depth), invariance of the whole step under a common shift
of all positions, and finite differences of the loss with respect to the unrotated Q and K; the
first-layer form with one shared key / value vector for all multi-token positions by finite differences
with respect to those vectors and by the K = 1 case.
Inference-side drafting: against the rows of the last anchor of the training-time problem (mask rebuilt
from the dependency rules), a library attention routine with an explicit mask, and the zero-query closed
form.  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "visible",
    "token_index",
    "token_coords",
    "element_mask",
    "attn_forward",
    "attn_backward",
    "segment_rows",
    "segment_keys",
    "attn_step_partitioned",
    "attn_step_partitioned_sampled",
    "cod_tokens",
    "packed_tokens",
    "partition_assign",
    "cod_position_count",
    "position_ids",
    "rope_angles",
    "rope_rotate",
    "attn_step_rope",
    "attn_step_rope_shared",
    "draft_decode",
]


# --------------------------------------------------------------------------------------
# index space and mask (Sec. 3: n x K positions; mask rule in the PARD paragraph and
# the dependency rule of Sec. 3.2, Challenge 2)
# --------------------------------------------------------------------------------------

def visible(i: int, d: int, j: int, e: int) -> bool:
    """May query (anchor i, depth d) attend to key (anchor j, depth e)?"""
    if e == 0:
        return j <= i
    return j == i and 1 <= e <= d


def token_index(i, d, L: int):
    """Depth-major storage order of the expanded sequence (blocks G0 | G1 | ... of Fig. 3)."""
    return d * L + i


def token_coords(t, L: int):
    """Inverse of :func:`token_index`: returns (anchor, depth)."""
    return t % L, t // L


def cod_tokens(depth_count: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Token list (anchor[t], depth[t]) of a drop-token sampled sequence in storage order:
    depth-major, each depth holding the anchors that keep it, ascending (anchor i keeps depths
    0 .. depth_count[i]-1)."""
    n = np.asarray(depth_count)
    assert (n >= 1).all()
    anchors, depths = [], []
    for g in range(int(n.max())):
        keep = np.nonzero(n > g)[0]
        anchors.append(keep)
        depths.append(np.full(len(keep), g))
    return np.concatenate(anchors), np.concatenate(depths)


def packed_tokens(seq_lens: Sequence[int], K: int, depth_count: Optional[Sequence[int]] = None):
    """Token list (anchor, depth, sequence) of a packed batch: the sequences are concatenated before the
    n x K expansion of Sec. 3, anchors are numbered across the batch, storage is depth-major over the
    whole batch (block G0 holds every sequence's depth-0 positions, then G1, ...).  ``depth_count``
    (per global anchor) selects a drop-token sample; default: every depth kept."""
    L = int(np.sum(seq_lens))
    n = np.full(L, K) if depth_count is None else np.asarray(depth_count)
    ta, td = cod_tokens(n)
    seq_of_anchor = np.repeat(np.arange(len(seq_lens)), seq_lens)
    return ta, td, seq_of_anchor[ta]


def element_mask(L: int, K: int, rows: Optional[np.ndarray] = None, cols: Optional[np.ndarray] = None,
                 tokens: Optional[Tuple[np.ndarray, np.ndarray]] = None) -> np.ndarray:
    """Boolean mask M[r, c] over expanded positions, evaluated element by element.

    ``rows`` / ``cols`` are token indices (default: all).  ``tokens`` gives the (anchor, depth)
    of every stored token for a sampled sequence; without it the sequence is dense, T = L*K.
    A third array in ``tokens`` is the sequence id of each token of a packed batch (anchors are
    then numbered across the whole batch): sequences do not see each other.
    """
    T = L * K if tokens is None else len(tokens[0])
    rows = np.arange(T) if rows is None else np.asarray(rows)
    cols = np.arange(T) if cols is None else np.asarray(cols)
    if tokens is None:
        i, d = token_coords(rows, L)
        j, e = token_coords(cols, L)
    else:
        ta, td = np.asarray(tokens[0]), np.asarray(tokens[1])
        i, d = ta[rows], td[rows]
        j, e = ta[cols], td[cols]
    i = i[:, None]
    d = d[:, None]
    j = j[None, :]
    e = e[None, :]
    depth0 = (e == 0) & (j <= i)
    if tokens is not None and len(tokens) == 3:
        ts = np.asarray(tokens[2])
        depth0 &= ts[rows][:, None] == ts[cols][None, :]
    chain = (e >= 1) & (e <= d) & (j == i)
    return depth0 | chain


# --------------------------------------------------------------------------------------
# dense masked attention, forward and backward
# --------------------------------------------------------------------------------------

def _row_blocks(rows: np.ndarray, block: int) -> Iterable[np.ndarray]:
    for s in range(0, len(rows), block):
        yield rows[s:s + block]


def _kv_head(h: int, Hq: int, Hkv: int) -> int:
    return h // (Hq // Hkv)


def attn_forward(q: np.ndarray, k: np.ndarray, v: np.ndarray, L: int, K: int, scale: float,
                 rows: Optional[np.ndarray] = None, cols: Optional[np.ndarray] = None,
                 row_block: int = 1024, return_probs: bool = False,
                 tokens: Optional[Tuple[np.ndarray, np.ndarray]] = None):
    """O = softmax(scale * Q K^T + mask) V and LSE = ln sum exp(scale * q.k) over visible keys.

    q: [T, Hq, D]; k, v: [T, Hkv, D] (fp64).  ``rows``: token indices of the query rows
    to compute (default all); ``cols``: token indices of the keys that are present
    (default all) - used by the segment semantics of Sec. 3.2.

    Returns O [len(rows), Hq, D], LSE [Hq, len(rows)] (and P [Hq, len(rows), len(cols)]
    when ``return_probs``).
    """
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert T == (L * K if tokens is None else len(tokens[0]))
    assert k.shape == v.shape and k.shape[0] == T and Hq % Hkv == 0
    rows = np.arange(T) if rows is None else np.asarray(rows)
    cols = np.arange(T) if cols is None else np.asarray(cols)
    O = np.zeros((len(rows), Hq, D), dtype=np.float64)
    LSE = np.zeros((Hq, len(rows)), dtype=np.float64)
    P_all = np.zeros((Hq, len(rows), len(cols)), dtype=np.float64) if return_probs else None
    pos = 0
    for rb in _row_blocks(rows, row_block):
        M = element_mask(L, K, rb, cols, tokens)
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            S = scale * (q[rb, h, :] @ k[cols, g, :].T)
            S = np.where(M, S, -np.inf)
            m = S.max(axis=1, keepdims=True)
            E = np.exp(S - m)
            Z = E.sum(axis=1, keepdims=True)
            P = E / Z
            O[pos:pos + len(rb), h, :] = P @ v[cols, g, :]
            LSE[h, pos:pos + len(rb)] = (m + np.log(Z))[:, 0]
            if return_probs:
                P_all[h, pos:pos + len(rb), :] = P
        pos += len(rb)
    if return_probs:
        return O, LSE, P_all
    return O, LSE


def attn_backward(q: np.ndarray, k: np.ndarray, v: np.ndarray, do: np.ndarray, L: int, K: int, scale: float,
                  rows: Optional[np.ndarray] = None, cols: Optional[np.ndarray] = None,
                  row_block: int = 1024, tokens: Optional[Tuple[np.ndarray, np.ndarray]] = None) -> Dict[str, np.ndarray]:
    """Gradients of sum(O * dO) for the rows in ``rows`` (default all).

    With P the softmax probabilities: dV = P^T dO, dP = dO V^T, Delta = rowsum(P * dP),
    dS = P * (dP - Delta), dQ = scale * dS K, dK = scale * dS^T Q; dK and dV are summed
    over the query heads that share a KV head.

    Returns dict with O, LSE, dQ (rows given, in the given order) and dK, dV
    ([T, Hkv, D], zero outside ``cols``).
    """
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    rows = np.arange(T) if rows is None else np.asarray(rows)
    cols = np.arange(T) if cols is None else np.asarray(cols)
    O = np.zeros((len(rows), Hq, D))
    LSE = np.zeros((Hq, len(rows)))
    dQ = np.zeros((len(rows), Hq, D))
    dK = np.zeros((T, Hkv, D))
    dV = np.zeros((T, Hkv, D))
    pos = 0
    for rb in _row_blocks(rows, row_block):
        M = element_mask(L, K, rb, cols, tokens)
        sl = slice(pos, pos + len(rb))
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            Kc = k[cols, g, :]
            Vc = v[cols, g, :]
            S = scale * (q[rb, h, :] @ Kc.T)
            S = np.where(M, S, -np.inf)
            m = S.max(axis=1, keepdims=True)
            E = np.exp(S - m)
            Z = E.sum(axis=1, keepdims=True)
            P = E / Z
            dOh = do[rb, h, :]
            O[sl, h, :] = P @ Vc
            LSE[h, sl] = (m + np.log(Z))[:, 0]
            dP = dOh @ Vc.T
            delta = (P * dP).sum(axis=1, keepdims=True)
            dS = P * (dP - delta)
            dQ[sl, h, :] = scale * (dS @ Kc)
            dK[cols, g, :] += scale * (dS.T @ q[rb, h, :])
            dV[cols, g, :] += P.T @ dOh
        pos += len(rb)
    return {"O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}


# --------------------------------------------------------------------------------------
# sequence partitioning / within-sequence gradient accumulation (Sec. 3.2)
# --------------------------------------------------------------------------------------

def segment_rows(L: int, K: int, b_lo: int, b_hi: int) -> np.ndarray:
    """Query rows of the segment holding anchors [b_lo, b_hi): every depth of those anchors."""
    i = np.arange(b_lo, b_hi)
    return np.concatenate([token_index(i, d, L) for d in range(K)])


def segment_keys(L: int, K: int, b_lo: int, b_hi: int) -> np.ndarray:
    """Keys present while the segment runs: depth-0 positions cumulatively up to the
    segment's end (Phase 3 of Algorithm 1) plus the segment's own positions."""
    n0 = np.arange(0, b_hi)                       # cumulative depth-0 context N_s
    own = np.arange(b_lo, b_hi)
    return np.concatenate([token_index(n0, 0, L)] + [token_index(own, d, L) for d in range(1, K)])


def attn_step_partitioned(q, k, v, do, L: int, K: int, scale: float, seg_bounds: Sequence[int],
                          row_block: int = 1024) -> Dict[str, np.ndarray]:
    """One forward+backward per segment, gradients accumulated across segments.

    Each segment runs as a separate pass that holds only its own rows and the keys of
    :func:`segment_keys`; dK and dV are summed over the passes in fp64; O, LSE and dQ
    of a row come from the one pass that owns the row.
    """
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    b = [int(x) for x in seg_bounds]
    assert b[0] == 0 and b[-1] == L and all(b[s] < b[s + 1] for s in range(len(b) - 1))
    O = np.zeros((T, Hq, D))
    LSE = np.zeros((Hq, T))
    dQ = np.zeros((T, Hq, D))
    dK = np.zeros((T, Hkv, D))
    dV = np.zeros((T, Hkv, D))
    for s in range(len(b) - 1):
        rows = segment_rows(L, K, b[s], b[s + 1])
        cols = segment_keys(L, K, b[s], b[s + 1])
        r = attn_backward(q, k, v, do, L, K, scale, rows=rows, cols=cols, row_block=row_block)
        O[rows] = r["O"]
        LSE[:, rows] = r["LSE"]
        dQ[rows] = r["dQ"]
        dK += r["dK"]
        dV += r["dV"]
    return {"O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}


def attn_step_partitioned_sampled(q, k, v, do, depth_count: Sequence[int], K: int, scale: float, S: int,
                                  row_block: int = 1024) -> Dict[str, np.ndarray]:
    """Within-sequence gradient accumulation for a drop-token sampled sequence, with the segment of
    every position taken from Algorithm 1 (:func:`partition_assign`) and each segment holding its
    own positions plus the cumulative depth-0 context N_s."""
    ta, td = cod_tokens(depth_count)
    L = len(depth_count)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    positions = [sorted((ta[td == g] + g).tolist()) for g in range(int(td.max()) + 1)]
    A, N = partition_assign(positions, S, L)
    seg_of_token = np.array([A[d][a + d] for a, d in zip(ta.tolist(), td.tolist())])
    tok_of = {(a, d): t for t, (a, d) in enumerate(zip(ta.tolist(), td.tolist()))}
    out = {"O": np.zeros((T, Hq, D)), "LSE": np.zeros((Hq, T)), "dQ": np.zeros((T, Hq, D)),
           "dK": np.zeros((T, Hkv, D)), "dV": np.zeros((T, Hkv, D))}
    for s in range(S):
        rows = np.nonzero(seg_of_token == s)[0]
        cols = np.array(sorted(set(rows.tolist()) | {tok_of[(p, 0)] for p in N[s]}))
        if len(rows) == 0:
            continue
        r = attn_backward(q, k, v, do, L, K, scale, rows=rows, cols=cols, row_block=row_block, tokens=(ta, td))
        out["O"][rows] = r["O"]
        out["LSE"][:, rows] = r["LSE"]
        out["dQ"][rows] = r["dQ"]
        out["dK"] += r["dK"]
        out["dV"] += r["dV"]
    return out


def partition_assign(positions: Sequence[Sequence[int]], S: int, L: int) -> Tuple[List[Dict[int, int]], List[List[int]]]:
    """Segment of every kept position (Algorithm 1; Sec. 3.2, Challenge 2) for possibly COD-sampled position sets.

    ``positions[g]`` lists the sequence positions kept at depth g.  The sequence is cut at s*L/S.  What must
    stay together is a dependency chain: position p at depth g needs position p-1 at depth g-1, and so on
    down to depth 1, so the chain through (p, g) starts at the depth-1 position p-g+1 and every member goes
    to the segment in which that head position lies.  Depth-0 positions go by their own position, and
    segment s also carries, as context, every depth-0 position before the cut that ends it.

    Returns (A, N): A[g] maps position -> segment, N[s] lists the cumulative depth-0 positions.
    """
    def segment_holding(position: int) -> int:          # the last cut at or before the position
        return max(s for s in range(S) if s * L / S <= position)

    kept = [set(ps) for ps in positions]
    A: List[Dict[int, int]] = [{p: segment_holding(p) for p in ps} for ps in positions[:1]]
    for g in range(1, len(positions)):
        A.append({})
        for p in positions[g]:
            head = p - (g - 1)                          # the chain's depth-1 member
            assert all(p - j in kept[g - j] for j in range(1, g)), "a kept position needs the chain below it"
            A[g][p] = segment_holding(head)
    N = [[p for p in positions[0] if p < (s + 1) * L / S] for s in range(S)]
    return A, N


def cod_position_count(n: int, K: int, r: float) -> float:
    """Total positions over all depths under geometric retention: n * (1 - r^K) / (1 - r) (Sec. 3.2)."""
    if r == 1.0:
        return float(n * K)
    return n * (1.0 - r ** K) / (1.0 - r)


# --------------------------------------------------------------------------------------
# rotary position embedding around the attention (Sec. 2: the drafter is a LLaMA 3 style
# decoder with RoPE, Su et al. 2024)
# --------------------------------------------------------------------------------------

def position_ids(L: int, K: int, tokens: Optional[Tuple[np.ndarray, ...]] = None) -> np.ndarray:
    """Sequence position of every stored token.  Depth d predicts the token d+1 ahead of its
    anchor (Sec. 3), so the row (anchor i, depth d) stands at position p = i + d - the same rows
    are written (p, d) in Sec. 3.2.  In a packed batch positions restart with every sequence."""
    if tokens is None:
        i, d = token_coords(np.arange(L * K), L)
        return i + d
    ta, td = np.asarray(tokens[0]), np.asarray(tokens[1])
    if len(tokens) == 3:
        ts = np.asarray(tokens[2])
        first = np.full(int(ts.max()) + 1, np.iinfo(np.int64).max)
        np.minimum.at(first, ts, ta)          # first anchor of each sequence
        return ta - first[ts] + td
    return ta + td


def rope_angles(pos: np.ndarray, D: int, base: float) -> np.ndarray:
    """angle[t, j] = pos[t] * base^(-2j/D), j = 0 .. D/2-1 (RoFormer, Eq. 15)."""
    j = np.arange(D // 2, dtype=np.float64)
    return np.asarray(pos, dtype=np.float64)[:, None] * np.float64(base) ** (-2.0 * j / D)


def rope_rotate(x: np.ndarray, pos: np.ndarray, base: float, inverse: bool = False) -> np.ndarray:
    """Rotate every head vector of x [T, H, D] by its token's position: the pair of features
    (j, j + D/2) turns by angle[t, j] (the half-split pairing of the LLaMA implementations; the
    paper names the architecture only).  ``inverse`` turns the other way (the transpose of the
    rotation, which is what gradients take)."""
    T, H, D = x.shape
    a = rope_angles(pos, D, base)
    c, s = np.cos(a)[:, None, :], np.sin(a)[:, None, :]
    if inverse:
        s = -s
    x1, x2 = x[..., :D // 2], x[..., D // 2:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def attn_step_rope(q, k, v, do, L: int, K: int, scale: float, seg_bounds: Sequence[int], base: float,
                   tokens: Optional[Tuple[np.ndarray, ...]] = None, pos: Optional[np.ndarray] = None,
                   row_block: int = 1024) -> Dict[str, np.ndarray]:
    """The attention step on unrotated Q and K: both are rotated by their positions, the attention
    runs on the rotated tensors, and dQ, dK come back with respect to the unrotated inputs (a rotation's
    Jacobian is the rotation itself, so each gradient vector is turned back).  Dense sequences run
    segment by segment (:func:`attn_step_partitioned`); an explicit token list runs as one pass
    (gradients do not depend on the partition).  ``pos`` overrides the position ids."""
    if pos is None:
        pos = position_ids(L, K, tokens)
    qr = rope_rotate(q, pos, base)
    kr = rope_rotate(k, pos, base)
    if tokens is None:
        r = attn_step_partitioned(qr, kr, v, do, L, K, scale, seg_bounds, row_block=row_block)
    else:
        r = attn_backward(qr, kr, v, do, L, K, scale, row_block=row_block, tokens=tokens)
    r = dict(r)
    r["dQ"] = rope_rotate(r["dQ"], pos, base, inverse=True)
    r["dK"] = rope_rotate(r["dK"], pos, base, inverse=True)
    return r


def attn_step_rope_shared(q, k0, k_shared, v0, v_shared, do, L: int, K: int, scale: float, seg_bounds: Sequence[int],
                          base: float, tokens: Optional[Tuple[np.ndarray, ...]] = None) -> Dict[str, np.ndarray]:
    """The step as the first drafter layer sees it (Sec. 2): every multi-token position (depth >= 1) is fed
    the same input - the shared hidden state and the mask-token embedding - so before the rotation all
    their keys are one vector per KV head, k_shared [Hkv, D], and all their values one vector v_shared;
    only the depth-0 positions (the first L stored tokens) have keys and values of their own, k0 / v0
    [L, Hkv, D].  Builds the full K and V, runs :func:`attn_step_rope`, and returns O, LSE, dQ as there,
    dK0 / dV0 for the depth-0 rows, and dK_shared / dV_shared: the sums over all chain positions (for the
    keys: of the gradients turned back to the unrotated frame)."""
    T = q.shape[0]
    Hkv, D = k_shared.shape
    assert k0.shape == (L, Hkv, D) and v0.shape == (L, Hkv, D) and v_shared.shape == (Hkv, D)
    k = np.concatenate([k0, np.broadcast_to(k_shared, (T - L, Hkv, D))], axis=0)
    v = np.concatenate([v0, np.broadcast_to(v_shared, (T - L, Hkv, D))], axis=0)
    r = attn_step_rope(q, k, v, do, L, K, scale, seg_bounds, base, tokens=tokens)
    return {"O": r["O"], "LSE": r["LSE"], "dQ": r["dQ"], "dK0": r["dK"][:L], "dV0": r["dV"][:L],
            "dK_shared": r["dK"][L:].sum(axis=0), "dV_shared": r["dV"][L:].sum(axis=0)}


# --------------------------------------------------------------------------------------
# inference-side parallel drafting (Sec. 2: all K draft tokens in one forward pass)
# --------------------------------------------------------------------------------------

def draft_decode(q_new: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, k_ctx: np.ndarray, v_ctx: np.ndarray,
                 scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Attention of one drafting step of one request.  The step adds K positions after a context of n
    tokens: the next-token position (depth 0, with real inputs) and K-1 multi-token positions (depths
    1..K-1), all belonging to the anchor n.  They are the rows (n, 0..K-1) of the parallel-prediction
    mask: row d sees the n context keys (depth-0 keys of earlier anchors, held in the KV cache), the
    new depth-0 key and its own chain, i.e. the new keys e <= d.

    q_new [K, Hq, D]; k_new, v_new [K, Hkv, D]; k_ctx, v_ctx [n, Hkv, D] (n may be 0).
    Returns O [K, Hq, D] and LSE [Hq, K] (natural log, scale included)."""
    K, Hq, D = q_new.shape
    Hkv = k_new.shape[1]
    n = k_ctx.shape[0]
    keys = np.concatenate([k_ctx, k_new], axis=0)
    vals = np.concatenate([v_ctx, v_new], axis=0)
    M = np.ones((K, n + K), dtype=bool)
    for d in range(K):
        for e in range(K):
            M[d, n + e] = visible(n, d, n, e)
    O = np.zeros((K, Hq, D))
    LSE = np.zeros((Hq, K))
    for h in range(Hq):
        g = _kv_head(h, Hq, Hkv)
        S = np.where(M, scale * (q_new[:, h, :] @ keys[:, g, :].T), -np.inf)
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        Z = E.sum(axis=1, keepdims=True)
        O[:, h, :] = (E / Z) @ vals[:, g, :]
        LSE[h] = (m + np.log(Z))[:, 0]
    return O, LSE
