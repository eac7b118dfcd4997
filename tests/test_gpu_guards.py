"""GPU tests: no entry point writes outside the buffers it was given.

Every output tensor and the workspace are carved out of a larger allocation with a guard region of a known
byte pattern on both sides; after the calls the guards must be unchanged.  The shapes have ragged tails (a
sequence length that is no multiple of a key tile or of a row tile's anchors, a row count below a tile)
because that is where a tile-granular kernel would overrun."""
import numpy as np
import pytest
import torch

import paper_2602_01469_amd as pe
from gpu_harness import rand_bits, to_dev_bf16
from peagle_inputs import make_decode_inputs

pytestmark = pytest.mark.gpu

GUARD = 8192          # bytes on each side
PATTERN = 0xA5


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


class Guarded:
    """Tensors of the requested shapes inside one byte buffer, each between two guard regions."""

    def __init__(self):
        self.items = []

    def tensor(self, name, shape, dtype):
        nbytes = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        padded = (nbytes + 255) // 256 * 256                       # the payload starts 256-byte aligned
        raw = torch.full((GUARD + padded + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        view = raw[GUARD:GUARD + nbytes].view(dtype).view(*shape)
        self.items.append((name, raw, nbytes))
        return view

    def check(self, what):
        torch.cuda.synchronize()
        for name, raw, nbytes in self.items:
            before = raw[:GUARD]
            after = raw[GUARD + nbytes:]
            assert bool((before == PATTERN).all()), f"{what}: bytes before {name} were written"
            assert bool((after == PATTERN).all()), f"{what}: bytes after {name} were written"


@pytest.mark.parametrize("L,K,Hq,Hkv,D,bounds", [
    (333, 8, 4, 2, 64, [0, 160, 333]),        # L % 64 = 13, L % 16 = 13
    (130, 4, 2, 1, 128, None),                # two anchors past a key tile, D = 128
    (77, 3, 3, 3, 64, None),                  # odd K: a row tile holds 126 rows
])
def test_training_step_stays_inside_its_buffers(L, K, Hq, Hkv, D, bounds):
    print(f"case guards step L={L} K={K} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    T = L * K
    q, do = to_dev_bf16(rand_bits((T, Hq, D), 900)), to_dev_bf16(rand_bits((T, Hq, D), 903))
    k, v = to_dev_bf16(rand_bits((T, Hkv, D), 901)), to_dev_bf16(rand_bits((T, Hkv, D), 902))
    tm = pe.peagle_build_tilemap(L, K, bounds, device=0)
    shape = pe.Shape(L, K, Hq, Hkv, D)
    S = 1 if bounds is None else len(bounds) - 1
    g = Guarded()
    o = g.tensor("o", (T, Hq, D), torch.bfloat16)
    dq = g.tensor("dq", (T, Hq, D), torch.bfloat16)
    lse = g.tensor("lse", (Hq, T), torch.float32)
    dk = g.tensor("dk_acc", (T, Hkv, D), torch.float32)
    dv = g.tensor("dv_acc", (T, Hkv, D), torch.float32)
    dkb = g.tensor("dk_bf16", (T, Hkv, D), torch.bfloat16)
    dvb = g.tensor("dv_bf16", (T, Hkv, D), torch.bfloat16)
    ws = g.tensor("workspace", (pe.peagle_workspace_bytes(tm, shape),), torch.uint8)
    pe.peagle_attn_step_partitioned(tm, shape, 0, S, q, k, v, do, o, lse, dq, dk, dv, dkb, dvb, ws)
    g.check("partitioned step")
    pe.peagle_attn_fwd(tm, shape, -1, q, k, v, o, lse)
    pe.peagle_attn_bwd(tm, shape, -1, q, k, v, o, do, lse, dq, dk, dv, 0, ws)
    g.check("unpartitioned forward + backward")
    assert torch.isfinite(o.float()).all() and torch.isfinite(dk).all()

    # the same problem with rotary embedding (rotated copies and the table live in the larger workspace)
    n_pos = pe.peagle_rope_positions(tm, L)
    g2 = Guarded()
    table = g2.tensor("rope_table", (n_pos, 2, D // 2), torch.float32)
    ws2 = g2.tensor("rope workspace", (pe.peagle_rope_workspace_bytes(tm, shape),), torch.uint8)
    pe.peagle_rope_table(500000.0, D, n_pos, table)
    pe.peagle_attn_step_partitioned_rope(tm, shape, 0, S, q, k, v, do, table, o, lse, dq, dk, dv, None, None, ws2)
    g.check("rotary step (outputs)")
    g2.check("rotary step (table, workspace)")


def test_sampled_and_packed_steps_stay_inside_their_buffers():
    from peagle_inputs import cod_depth_counts
    print("case guards sampled / packed", flush=True)
    K, Hq, Hkv, D = 8, 4, 2, 64
    seq_lens = [150, 77, 201]
    counts = np.concatenate([cod_depth_counts(n, K, 0.8, 950 + i) for i, n in enumerate(seq_lens)])
    tm = pe.peagle_build_tilemap_packed(seq_lens, K, counts, [0, 227, sum(seq_lens)], device=0)
    L = sum(seq_lens)
    T = tm.tokens(L)
    shape = pe.Shape(L, K, Hq, Hkv, D)
    q, do = to_dev_bf16(rand_bits((T, Hq, D), 960)), to_dev_bf16(rand_bits((T, Hq, D), 963))
    k, v = to_dev_bf16(rand_bits((T, Hkv, D), 961)), to_dev_bf16(rand_bits((T, Hkv, D), 962))
    g = Guarded()
    o = g.tensor("o", (T, Hq, D), torch.bfloat16)
    dq = g.tensor("dq", (T, Hq, D), torch.bfloat16)
    lse = g.tensor("lse", (Hq, T), torch.float32)
    dk = g.tensor("dk_acc", (T, Hkv, D), torch.float32)
    dv = g.tensor("dv_acc", (T, Hkv, D), torch.float32)
    ws = g.tensor("workspace", (pe.peagle_workspace_bytes(tm, shape),), torch.uint8)
    pe.peagle_attn_step_partitioned(tm, shape, 0, 2, q, k, v, do, o, lse, dq, dk, dv, None, None, ws)
    g.check("packed sampled step")
    assert torch.isfinite(dq.float()).all()


def test_drafting_step_stays_inside_its_buffers():
    print("case guards decode", flush=True)
    K, Hq, Hkv, D = 5, 12, 4, 64                # 15 query rows per KV head: half a row block
    inp = make_decode_inputs((130, 0, 63, 1000), K, Hq, Hkv, D, 970)
    C = len(inp["ctx_len"])
    shape = pe.DecodeShape(C, K, Hq, Hkv, D, inp["n_pages"], inp["max_pages"], None)
    q, k, v = (to_dev_bf16(inp[n]) for n in ("q_new", "k_new", "v_new"))
    kp, vp = to_dev_bf16(inp["k_pages"]), to_dev_bf16(inp["v_pages"])
    bt, cl = torch.from_numpy(inp["block_table"]).cuda(), torch.from_numpy(inp["ctx_len"]).cuda()
    g = Guarded()
    o = g.tensor("o", (C, K, Hq, D), torch.bfloat16)
    lse = g.tensor("lse", (C, Hq, K), torch.float32)
    status = g.tensor("status", (C,), torch.int32)
    ws = g.tensor("workspace", (pe.peagle_draft_decode_workspace_bytes(shape),), torch.uint8)
    pe.peagle_draft_decode(shape, q, k, v, kp, vp, bt, cl, o, lse, status, ws)
    g.check("drafting step")
    pe.peagle_draft_decode_static(shape, q, k, v, kp, vp, bt, cl, o, lse, status)
    g.check("drafting step, static scratch")
    assert torch.isfinite(o.float()).all() and (status == 0).all()
