"""Workload shapes and seeded bf16 tensors for the parallel-drafting attention path.

The paper's long-context training traces (sequence-length quantiles in its Fig. 1:
median about 3.9k, P90 about 10.8k, P99 about 20k tokens) and drafter head shapes
are not available offline, so synthetic tensors of the same shapes stand in for them.

Recipe (identical for every consumer):
  * ``numpy.random.default_rng(seed)``;
  * fp32 ``standard_normal`` draws in the order Q, K, V, dO, each in its final
    ``[T, H, D]`` shape (``T = L*K`` expanded positions, depth-major ``t = d*L + i``);
  * multiply by ``value_scale`` (0.5 for the P99 stress case, else 1);
  * round to nearest even to bf16; the uint16 bit patterns are the inputs.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    L: int            # anchor tokens (sequence length n of the paper, Sec. 3)
    K: int            # parallel prediction depths
    Hq: int
    Hkv: int
    D: int
    seed: int
    seg_anchors: int  # anchors per query-row segment (Sec. 3.2); 0 = single segment
    value_scale: float = 1.0

    @property
    def T(self) -> int:
        return self.L * self.K

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    def seg_bounds(self) -> np.ndarray:
        """Anchor boundaries b_0=0 < ... < b_S=L of the query-row segments."""
        if self.seg_anchors <= 0 or self.seg_anchors >= self.L:
            return np.array([0, self.L], dtype=np.int32)
        b = list(range(0, self.L, self.seg_anchors)) + [self.L]
        return np.array(b, dtype=np.int32)


CONFIGS: Dict[str, WorkloadConfig] = {
    "c1_tiny": WorkloadConfig("c1_tiny", L=128, K=4, Hq=4, Hkv=1, D=64, seed=0, seg_anchors=0),
    "c2_gptoss": WorkloadConfig("c2_gptoss", L=2048, K=4, Hq=64, Hkv=8, D=64, seed=1, seg_anchors=0),
    "c3_median": WorkloadConfig("c3_median", L=4096, K=8, Hq=64, Hkv=8, D=64, seed=2, seg_anchors=1024),
    "c4_p90": WorkloadConfig("c4_p90", L=10816, K=8, Hq=32, Hkv=4, D=128, seed=3, seg_anchors=2048),
    "c5_p99": WorkloadConfig("c5_p99", L=20480, K=8, Hq=64, Hkv=8, D=64, seed=4, seg_anchors=2048, value_scale=0.5),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def make_inputs(cfg: WorkloadConfig, L: int | None = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """bf16 bit patterns (uint16) of Q [T,Hq,D], K [T,Hkv,D], V [T,Hkv,D], dO [T,Hq,D].

    ``L`` overrides the anchor count (same seed and draw order) for reduced-size cases.
    """
    L = cfg.L if L is None else int(L)
    T = L * cfg.K
    rng = np.random.default_rng(cfg.seed)
    out = []
    for H in (cfg.Hq, cfg.Hkv, cfg.Hkv, cfg.Hq):
        x = rng.standard_normal(size=(T, H, cfg.D), dtype=np.float32)
        if cfg.value_scale != 1.0:
            x *= np.float32(cfg.value_scale)
        out.append(f32_to_bf16_bits(x))
        del x
    q, k, v, do = out
    return q, k, v, do


def useful_pairs(L: int, K: int) -> int:
    """Unmasked (row, key) pairs per query head: K*L*(L+1)/2 causal depth-0 pairs + L*K*(K-1)/2 chain pairs."""
    return K * L * (L + 1) // 2 + L * K * (K - 1) // 2


def useful_flops(L: int, K: int, Hq: int, D: int) -> int:
    """Forward 4*D and backward 10*D flops per unmasked pair per query head."""
    return 14 * D * Hq * useful_pairs(L, K)


def cod_depth_counts(L: int, K: int, retention: float, seed: int) -> np.ndarray:
    """Depths kept per anchor under Conditional Drop-token sampling (PARD paragraph of the paper's
    Sec. 3): depth 0 keeps all L positions, depth g keeps round(retention * |depth g-1|) of the
    anchors kept at depth g-1, chosen uniformly at random (a position needs its predecessor at the
    previous depth, so the kept sets are nested per anchor).  Returns int32[L] with values in 1..K."""
    rng = np.random.default_rng(seed)
    count = np.ones(L, dtype=np.int32)
    alive = np.arange(L)
    for g in range(1, K):
        n_keep = int(round(retention * len(alive)))
        if n_keep == 0:
            break
        alive = np.sort(rng.choice(alive, size=n_keep, replace=False))
        count[alive] = g + 1
    return count


def make_inputs_tokens(cfg: WorkloadConfig, T: int, seed_offset: int = 1000):
    """Q, K, V, dO bit patterns for a sequence of T stored tokens (sampled layouts), same recipe as make_inputs."""
    rng = np.random.default_rng(cfg.seed + seed_offset)
    out = []
    for H in (cfg.Hq, cfg.Hkv, cfg.Hkv, cfg.Hq):
        x = rng.standard_normal(size=(T, H, cfg.D), dtype=np.float32)
        if cfg.value_scale != 1.0:
            x *= np.float32(cfg.value_scale)
        out.append(f32_to_bf16_bits(x))
    return tuple(out)


def useful_pairs_sampled(depth_count) -> int:
    """Unmasked (query, key) pairs of a sampled sequence: the row of anchor i at depth d sees i+1 depth-0
    keys and d chain keys, and anchor i keeps depths 0..depth_count[i]-1."""
    n = np.asarray(depth_count, dtype=np.int64)
    i = np.arange(len(n), dtype=np.int64)
    return int((n * (i + 1) + n * (n - 1) // 2).sum())


PAGE_TOKENS = 64


def make_decode_inputs(ctx_lens, K: int, Hq: int, Hkv: int, D: int, seed: int, spare_pages: int = 3,
                       value_scale: float = 1.0):
    """Inputs of one inference-side drafting step for C = len(ctx_lens) requests (the serving setting of the
    paper: K = 3, 5, 7 draft positions, concurrency 2-4).  Returns bf16 bit patterns:

      q_new [C, K, Hq, D], k_new / v_new [C, K, Hkv, D];
      k_ctx / v_ctx: per request, [n_c, Hkv, D] (what the oracle reads);
      k_pages / v_pages [n_pages, Hkv, 64, D], block_table [C, max_pages] int32, ctx_len [C] int32
      (what the HIP path reads: the same context tokens scattered over a shuffled page pool; unused
      table entries are -1 and the unused tail of every last page holds NaN bit patterns, as
      uninitialised cache memory might).
    """
    rng = np.random.default_rng(seed)
    C = len(ctx_lens)
    draw = lambda shape: f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(value_scale))
    q_new, k_new, v_new = draw((C, K, Hq, D)), draw((C, K, Hkv, D)), draw((C, K, Hkv, D))
    k_ctx = [draw((int(n), Hkv, D)) for n in ctx_lens]
    v_ctx = [draw((int(n), Hkv, D)) for n in ctx_lens]
    pages_of = [(int(n) + PAGE_TOKENS - 1) // PAGE_TOKENS for n in ctx_lens]
    max_pages = max(1, max(pages_of))
    n_pages = max(1, sum(pages_of) + spare_pages)
    perm = rng.permutation(n_pages)
    k_pages = np.full((n_pages, Hkv, PAGE_TOKENS, D), 0x7FC0, dtype=np.uint16)   # bf16 NaN
    v_pages = np.full((n_pages, Hkv, PAGE_TOKENS, D), 0x7FC0, dtype=np.uint16)
    block_table = np.full((C, max_pages), -1, dtype=np.int32)
    nxt = 0
    for c, n in enumerate(ctx_lens):
        for b in range(pages_of[c]):
            page = int(perm[nxt])
            nxt += 1
            block_table[c, b] = page
            lo, hi = b * PAGE_TOKENS, min(int(n), (b + 1) * PAGE_TOKENS)
            k_pages[page, :, :hi - lo] = k_ctx[c][lo:hi].transpose(1, 0, 2)
            v_pages[page, :, :hi - lo] = v_ctx[c][lo:hi].transpose(1, 0, 2)
    return {"q_new": q_new, "k_new": k_new, "v_new": v_new, "k_ctx": k_ctx, "v_ctx": v_ctx, "k_pages": k_pages,
            "v_pages": v_pages, "block_table": block_table, "ctx_len": np.asarray(ctx_lens, dtype=np.int32),
            "n_pages": n_pages, "max_pages": max_pages}
