"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding on seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import paper_2602_01469_amd as pe
from peagle_inputs import bf16_bits_to_f64


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return bf16_bits_to_f64(t.view(torch.int16).cpu().numpy().view(np.uint16))


def rand_bits(shape, seed, scale=1.0):
    from peagle_inputs import f32_to_bf16_bits
    rng = np.random.default_rng(seed)
    return f32_to_bf16_bits((rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)))


class Run:
    """Device buffers of one problem and the calls that fill them."""

    def __init__(self, tm, L, K, Hq, Hkv, D, qb, kb, vb, dob, scale=None):
        self.tm = tm
        self.shape = pe.Shape(L, K, Hq, Hkv, D, scale)
        T = L * K
        self.q, self.k, self.v, self.do = (to_dev_bf16(x) for x in (qb, kb, vb, dob))
        self.o = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        self.dq = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        self.lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
        self.dk = torch.full((T, Hkv, D), float("nan"), dtype=torch.float32, device="cuda")
        self.dv = torch.full((T, Hkv, D), float("nan"), dtype=torch.float32, device="cuda")
        self.ws = torch.empty(pe.peagle_workspace_bytes(tm, self.shape), dtype=torch.uint8, device="cuda")

    def fwd(self, seg=-1):
        pe.peagle_attn_fwd(self.tm, self.shape, seg, self.q, self.k, self.v, self.o, self.lse)

    def bwd(self, seg=-1, accumulate=0):
        pe.peagle_attn_bwd(self.tm, self.shape, seg, self.q, self.k, self.v, self.o, self.do, self.lse, self.dq,
                           self.dk, self.dv, accumulate, self.ws)

    def step(self, seg_begin, seg_end, dk_bf16=None, dv_bf16=None):
        pe.peagle_attn_step_partitioned(self.tm, self.shape, seg_begin, seg_end, self.q, self.k, self.v, self.do,
                                        self.o, self.lse, self.dq, self.dk, self.dv, dk_bf16, dv_bf16, self.ws)

    def results(self):
        torch.cuda.synchronize()
        return {"O": bf16_to_f64(self.o), "LSE": self.lse.double().cpu().numpy(), "dQ": bf16_to_f64(self.dq),
                "dK": self.dk.double().cpu().numpy(), "dV": self.dv.double().cpu().numpy()}


class SampledRun(Run):
    """Same for a drop-token sampled sequence: `tm` is a sampled tile map, T = its kept positions."""

    def __init__(self, tm, L, K, Hq, Hkv, D, qb, kb, vb, dob, scale=None):
        self.tm = tm
        self.shape = pe.Shape(L, K, Hq, Hkv, D, scale)
        T = tm.tokens(L)
        assert qb.shape[0] == T
        self.q, self.k, self.v, self.do = (to_dev_bf16(x) for x in (qb, kb, vb, dob))
        self.o = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        self.dq = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        self.lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
        self.dk = torch.full((T, Hkv, D), float("nan"), dtype=torch.float32, device="cuda")
        self.dv = torch.full((T, Hkv, D), float("nan"), dtype=torch.float32, device="cuda")
        self.ws = torch.empty(pe.peagle_workspace_bytes(tm, self.shape), dtype=torch.uint8, device="cuda")


def rel_l2(a, b):
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


def max_abs(a, b):
    return float(np.abs(a - b).max())


def attach_rope(run, base):
    """Adds a rotary table and the larger workspace to a Run / SampledRun; returns run.step_rope."""
    L, D = run.shape.L, run.shape.D
    n_pos = pe.peagle_rope_positions(run.tm, L)
    run.rope_table = torch.full((n_pos, 2, D // 2), float("nan"), dtype=torch.float32, device="cuda")
    pe.peagle_rope_table(base, D, n_pos, run.rope_table)
    run.ws = torch.empty(pe.peagle_rope_workspace_bytes(run.tm, run.shape), dtype=torch.uint8, device="cuda")

    def step_rope(seg_begin, seg_end, dk_bf16=None, dv_bf16=None):
        pe.peagle_attn_step_partitioned_rope(run.tm, run.shape, seg_begin, seg_end, run.q, run.k, run.v, run.do,
                                             run.rope_table, run.o, run.lse, run.dq, run.dk, run.dv, dk_bf16, dv_bf16,
                                             run.ws)
    run.step_rope = step_rope
    return run
