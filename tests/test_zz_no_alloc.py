"""GPU test of peagle_draft_decode_static, the drafting step for callers that cannot allocate (its partial
records live in an array inside the library instead of a caller workspace).  It is called through the C ABI
twice in a row, the second time on a smaller batch, and each result is compared with peagle_draft_decode on
the same inputs (same kernels and launch shapes: identical bits) and with the fp64 oracle at the forward's
tolerances (O rel-L2 <= 5e-3, max-abs <= 1e-2 where the bf16 output format allows, LSE <= 4e-3)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2602_01469_amd as pe
from gpu_harness import bf16_to_f64
from peagle_inputs import make_decode_inputs
from test_gpu_decode import DecodeRun, _check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _static_call(r):
    """peagle_draft_decode_static through the raw C ABI (ctypes), on the buffers of a DecodeRun."""
    lib = pe.load_library()
    s = r.shape
    r.o.fill_(float("nan"))
    r.lse.fill_(float("nan"))
    r.status.fill_(-7)
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = lib.peagle_draft_decode_static(s.c(), p(r.q), p(r.k), p(r.v), p(r.kp), p(r.vp), p(r.bt), p(r.cl), p(r.o),
                                        p(r.lse), p(r.status), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, pe.peagle_strerror(rc)
    torch.cuda.synchronize()
    return bf16_to_f64(r.o), r.lse.double().cpu().numpy(), r.status.cpu().numpy()


CALLS = [
    # ctx_lens, K, Hq, Hkv, D, seed: a batch with many splits first, then a smaller one that leaves most of the
    # first call's records in the array untouched
    ((4096, 1500, 333, 2048), 7, 64, 8, 64, 2000),
    ((300, 70), 3, 16, 2, 64, 2010),
]


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    for ctx_lens, K, Hq, Hkv, D, seed in CALLS:
        print(f"case decode static: ctx={ctx_lens} K={K} Hq={Hq} Hkv={Hkv} D={D} seed={seed}", flush=True)
        inp = make_decode_inputs(ctx_lens, K, Hq, Hkv, D, seed)
        r = DecodeRun(inp, K, Hq, Hkv, D)
        o_ws, lse_ws, st_ws = r.run()
        o_st, lse_st, st_st = _static_call(r)
        assert (st_st == 0).all() and np.array_equal(st_st, st_ws)
        assert np.array_equal(o_st, o_ws) and np.array_equal(lse_st, lse_ws)
        _check(inp, o_st, lse_st, r.shape.scale, f"static {ctx_lens}")


def test_static_scratch_entry_point_rejects_shapes_beyond_its_array():
    """Records of 4,096 requests x 8 KV heads do not fit the array: refused before any launch, outputs untouched."""
    print("case decode static: oversized shape", flush=True)
    shape = pe.DecodeShape(4096, 7, 64, 8, 64, 8, 1)
    assert pe.peagle_draft_decode_workspace_bytes(shape) > 32 << 20
    lib = pe.load_library()
    one = C.c_void_p(256)  # never dereferenced: the size check comes before any launch
    rc = lib.peagle_draft_decode_static(shape.c(), one, one, one, one, one, one, one, one, one, None, None)
    assert rc == -6, rc  # PEAGLE_EWORKSPACE
