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
