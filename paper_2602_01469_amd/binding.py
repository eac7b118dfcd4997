"""ctypes binding: argument marshalling only.  Names mirror the C ABI of include/peagle.h."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libpeagle_attn.so"
_lib = None


class PeagleError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {peagle_strerror(status)} (status {status})")


class _ShapeC(C.Structure):
    _fields_ = [("L", C.c_int32), ("K", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("layout", C.c_int32), ("scale", C.c_float)]


class _InfoC(C.Structure):
    _fields_ = [("L_max", C.c_int32), ("K", C.c_int32), ("S", C.c_int32), ("anchors_per_row_tile", C.c_int32),
                ("rows_per_tile", C.c_int32), ("keys_per_tile", C.c_int32), ("n_row_tiles", C.c_int32),
                ("n_depth0_key_tiles", C.c_int32), ("n_chain_sub_tiles", C.c_int32), ("n_key_tiles", C.c_int32),
                ("n_full", C.c_int64), ("n_partial", C.c_int64), ("n_masks", C.c_int32), ("device_bytes", C.c_int64),
                ("tokens", C.c_int64), ("sampled", C.c_int32)]


class _DecodeShapeC(C.Structure):
    _fields_ = [("C", C.c_int32), ("K", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("scale", C.c_float), ("n_pages", C.c_int32), ("max_pages", C.c_int32)]


EXPORTS = [
    "peagle_build_tilemap", "peagle_tilemap_destroy", "peagle_tilemap_info", "peagle_tilemap_expand_rows",
    "peagle_tilemap_classes", "peagle_workspace_bytes", "peagle_attn_fwd", "peagle_attn_bwd",
    "peagle_attn_step_partitioned", "peagle_build_tilemap_sampled", "peagle_build_tilemap_packed",
    "peagle_tilemap_rebuild", "peagle_tilemap_tokens",
    "peagle_rope_positions", "peagle_rope_position_ids", "peagle_rope_table", "peagle_rope_rotate", "peagle_rope_workspace_bytes",
    "peagle_attn_step_partitioned_rope", "peagle_attn_step_rope_profiled",
    "peagle_rope_shared_workspace_bytes", "peagle_attn_step_rope_shared",
    "peagle_draft_decode_splits", "peagle_draft_decode_workspace_bytes", "peagle_draft_decode",
    "peagle_draft_decode_static",
    "peagle_attn_step_profiled", "peagle_measure_mfma_ceiling", "peagle_measure_mfma_ceiling_random", "peagle_device_info", "peagle_strerror",
]

KERNEL_KINDS = ("fwd", "dq", "dkdv", "reduce", "rope")


class _ProfileC(C.Structure):
    _fields_ = [("ms", C.c_float * len(KERNEL_KINDS)), ("launches", C.c_int32 * len(KERNEL_KINDS))]


def lib_path() -> str:
    """The in-tree build; PEAGLE_ATTN_LIB names another build of the same sources (the host-sanitizer test's)."""
    return os.environ.get("PEAGLE_ATTN_LIB") or os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load the HIP extension; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2602_01469_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    lib.peagle_build_tilemap.argtypes = [i32, i32, C.POINTER(i32), i32, i32, C.POINTER(vp)]
    lib.peagle_build_tilemap.restype = C.c_int
    lib.peagle_tilemap_destroy.argtypes = [vp]
    lib.peagle_tilemap_destroy.restype = None
    lib.peagle_tilemap_info.argtypes = [vp, C.POINTER(_InfoC)]
    lib.peagle_tilemap_info.restype = C.c_int
    lib.peagle_tilemap_expand_rows.argtypes = [vp, i32, i32, i64, i64, vp]
    lib.peagle_tilemap_expand_rows.restype = C.c_int
    lib.peagle_tilemap_classes.argtypes = [vp, vp]
    lib.peagle_tilemap_classes.restype = C.c_int
    lib.peagle_workspace_bytes.argtypes = [vp, C.POINTER(_ShapeC)]
    lib.peagle_workspace_bytes.restype = sz
    lib.peagle_attn_fwd.argtypes = [vp, C.POINTER(_ShapeC), i32, vp, vp, vp, vp, vp, vp]
    lib.peagle_attn_fwd.restype = C.c_int
    lib.peagle_attn_bwd.argtypes = [vp, C.POINTER(_ShapeC), i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.peagle_attn_bwd.restype = C.c_int
    lib.peagle_attn_step_partitioned.argtypes = [vp, C.POINTER(_ShapeC), i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                 vp, vp, vp, sz, vp]
    lib.peagle_attn_step_partitioned.restype = C.c_int
    lib.peagle_build_tilemap_sampled.argtypes = [C.POINTER(i32), i32, i32, C.POINTER(i32), i32, i32, i32,
                                                 C.POINTER(vp)]
    lib.peagle_build_tilemap_sampled.restype = C.c_int
    lib.peagle_build_tilemap_packed.argtypes = [C.POINTER(i32), i32, i32, C.POINTER(i32), i32, C.POINTER(i32), i32,
                                                i32, i32, C.POINTER(vp)]
    lib.peagle_build_tilemap_packed.restype = C.c_int
    lib.peagle_tilemap_rebuild.argtypes = [vp, C.POINTER(i32), i32, C.POINTER(i32), i32, C.POINTER(i32), i32, i32, vp]
    lib.peagle_tilemap_rebuild.restype = C.c_int
    lib.peagle_tilemap_tokens.argtypes = [vp, i32]
    lib.peagle_tilemap_tokens.restype = i64
    lib.peagle_attn_step_profiled.argtypes = [vp, C.POINTER(_ShapeC), i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                              sz, vp, C.POINTER(_ProfileC)]
    lib.peagle_attn_step_profiled.restype = C.c_int
    lib.peagle_rope_positions.argtypes = [vp, i32]
    lib.peagle_rope_positions.restype = i32
    lib.peagle_rope_position_ids.argtypes = [vp, i32, C.POINTER(i32)]
    lib.peagle_rope_position_ids.restype = C.c_int
    lib.peagle_rope_table.argtypes = [C.c_float, i32, i32, vp, vp]
    lib.peagle_rope_table.restype = C.c_int
    lib.peagle_rope_rotate.argtypes = [vp, C.POINTER(_ShapeC), vp, i32, vp, i32, i32, vp, vp]
    lib.peagle_rope_rotate.restype = C.c_int
    lib.peagle_rope_workspace_bytes.argtypes = [vp, C.POINTER(_ShapeC)]
    lib.peagle_rope_workspace_bytes.restype = sz
    lib.peagle_attn_step_partitioned_rope.argtypes = [vp, C.POINTER(_ShapeC), i32, i32, vp, vp, vp, vp, vp, i32, vp, vp,
                                                      vp, vp, vp, vp, vp, vp, sz, vp]
    lib.peagle_attn_step_partitioned_rope.restype = C.c_int
    lib.peagle_attn_step_rope_profiled.argtypes = [vp, C.POINTER(_ShapeC), i32, i32, vp, vp, vp, vp, vp, i32, vp, vp,
                                                   vp, vp, vp, vp, sz, vp, C.POINTER(_ProfileC)]
    lib.peagle_attn_step_rope_profiled.restype = C.c_int
    lib.peagle_rope_shared_workspace_bytes.argtypes = [vp, C.POINTER(_ShapeC)]
    lib.peagle_rope_shared_workspace_bytes.restype = sz
    lib.peagle_attn_step_rope_shared.argtypes = [vp, C.POINTER(_ShapeC), vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp,
                                                 vp, vp, vp, vp, sz, vp]
    lib.peagle_attn_step_rope_shared.restype = C.c_int
    lib.peagle_draft_decode_splits.argtypes = [C.POINTER(_DecodeShapeC)]
    lib.peagle_draft_decode_splits.restype = i32
    lib.peagle_draft_decode_workspace_bytes.argtypes = [C.POINTER(_DecodeShapeC)]
    lib.peagle_draft_decode_workspace_bytes.restype = sz
    lib.peagle_draft_decode.argtypes = [C.POINTER(_DecodeShapeC), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.peagle_draft_decode.restype = C.c_int
    lib.peagle_draft_decode_static.argtypes = [C.POINTER(_DecodeShapeC), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.peagle_draft_decode_static.restype = C.c_int
    lib.peagle_measure_mfma_ceiling.argtypes = [vp, C.POINTER(C.c_float)]
    lib.peagle_measure_mfma_ceiling.restype = C.c_int
    lib.peagle_measure_mfma_ceiling_random.argtypes = [vp, C.POINTER(C.c_float)]
    lib.peagle_measure_mfma_ceiling_random.restype = C.c_int
    lib.peagle_device_info.argtypes = [C.POINTER(i32), C.POINTER(i32)]
    lib.peagle_device_info.restype = C.c_int
    lib.peagle_strerror.argtypes = [C.c_int]
    lib.peagle_strerror.restype = C.c_char_p
    _lib = lib
    return lib


def peagle_strerror(status: int) -> str:
    return load_library().peagle_strerror(int(status)).decode()


class Shape:
    """Mirror of peagle_shape_t."""

    def __init__(self, L: int, K: int, Hq: int, Hkv: int, D: int, scale: Optional[float] = None, layout: int = 0):
        self.L, self.K, self.Hq, self.Hkv, self.D, self.layout = int(L), int(K), int(Hq), int(Hkv), int(D), int(layout)
        self.scale = float(scale) if scale is not None else 1.0 / float(np.sqrt(D))
        self._c = _ShapeC(self.L, self.K, self.Hq, self.Hkv, self.D, self.layout, self.scale)

    @property
    def T(self) -> int:
        return self.L * self.K

    def c(self):
        return C.byref(self._c)


class TileMap:
    """Owner of a peagle_tilemap_t handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)

    @property
    def handle(self):
        if not self._h:
            raise ValueError("tile map already destroyed")
        return self._h

    def destroy(self):
        if self._h:
            load_library().peagle_tilemap_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def info(self) -> dict:
        inf = _InfoC()
        rc = load_library().peagle_tilemap_info(self.handle, C.byref(inf))
        if rc != 0:
            raise PeagleError(rc, "peagle_tilemap_info")
        return {name: getattr(inf, name) for name, _ in _InfoC._fields_}

    def tokens(self, L: int) -> int:
        """Stored tokens T of a length-L sequence under this map (L*K, or the kept positions of a sampled map)."""
        T = int(load_library().peagle_tilemap_tokens(self.handle, int(L)))
        if T < 0:
            raise PeagleError(-3, "peagle_tilemap_tokens")
        return T

    def rebuild(self, seq_lens: Sequence[int], depth_count: Optional[Sequence[int]] = None,
                seg_bounds: Optional[Sequence[int]] = None, assignment: int = 0, stream=None) -> None:
        """peagle_tilemap_rebuild: new position set for a sampled / packed map, in place."""
        i32p = C.POINTER(C.c_int32)
        start = np.ascontiguousarray(np.concatenate([[0], np.cumsum(seq_lens)]), dtype=np.int32)
        L = int(start[-1])
        n = None if depth_count is None else np.ascontiguousarray(depth_count, dtype=np.int32)
        if n is not None and len(n) != L:
            raise ValueError("depth_count must have one entry per anchor of the batch")
        b = None if seg_bounds is None else np.ascontiguousarray(seg_bounds, dtype=np.int32)
        sp = None
        if self.info()["device_bytes"] > 0:
            sp = _stream_ptr(stream)
        rc = load_library().peagle_tilemap_rebuild(
            self.handle, None if n is None else n.ctypes.data_as(i32p), L, start.ctypes.data_as(i32p), len(start) - 1,
            None if b is None else b.ctypes.data_as(i32p), 1 if b is None else len(b) - 1, assignment, sp)
        if rc != 0:
            raise PeagleError(rc, "peagle_tilemap_rebuild")

    def expand_rows(self, L: int, seg: int, row_begin: int, row_end: int) -> np.ndarray:
        """Packed element-mask bits [row_end-row_begin, ceil(T/8)] (uint8, little bit order)."""
        row_bytes = (self.tokens(L) + 7) // 8
        out = np.zeros((max(row_end - row_begin, 0), row_bytes), dtype=np.uint8)
        rc = load_library().peagle_tilemap_expand_rows(self.handle, L, seg, row_begin, row_end,
                                                       out.ctypes.data_as(C.c_void_p))
        if rc != 0:
            raise PeagleError(rc, "peagle_tilemap_expand_rows")
        return out

    def classes(self) -> np.ndarray:
        inf = self.info()
        out = np.zeros((inf["n_row_tiles"], inf["n_key_tiles"]), dtype=np.uint8)
        rc = load_library().peagle_tilemap_classes(self.handle, out.ctypes.data_as(C.c_void_p))
        if rc != 0:
            raise PeagleError(rc, "peagle_tilemap_classes")
        return out


def peagle_build_tilemap(L_max: int, K: int, seg_bounds: Optional[Sequence[int]] = None, device: int = 0) -> TileMap:
    lib = load_library()
    out = C.c_void_p()
    if seg_bounds is None:
        rc = lib.peagle_build_tilemap(L_max, K, None, 1, device, C.byref(out))
    else:
        b = np.ascontiguousarray(seg_bounds, dtype=np.int32)
        rc = lib.peagle_build_tilemap(L_max, K, b.ctypes.data_as(C.POINTER(C.c_int32)), len(b) - 1, device,
                                      C.byref(out))
    if rc != 0:
        raise PeagleError(rc, "peagle_build_tilemap")
    return TileMap(out.value)


ASSIGN_BY_ANCHOR, ASSIGN_ALGORITHM1 = 0, 1


def peagle_build_tilemap_sampled(depth_count: Sequence[int], K: int, seg_bounds: Optional[Sequence[int]] = None,
                                 device: int = 0, assignment: int = ASSIGN_BY_ANCHOR) -> TileMap:
    lib = load_library()
    n = np.ascontiguousarray(depth_count, dtype=np.int32)
    out = C.c_void_p()
    if seg_bounds is None:
        rc = lib.peagle_build_tilemap_sampled(n.ctypes.data_as(C.POINTER(C.c_int32)), len(n), K, None, 1, assignment,
                                              device, C.byref(out))
    else:
        b = np.ascontiguousarray(seg_bounds, dtype=np.int32)
        rc = lib.peagle_build_tilemap_sampled(n.ctypes.data_as(C.POINTER(C.c_int32)), len(n), K,
                                              b.ctypes.data_as(C.POINTER(C.c_int32)), len(b) - 1, assignment, device,
                                              C.byref(out))
    if rc != 0:
        raise PeagleError(rc, "peagle_build_tilemap_sampled")
    return TileMap(out.value)


def peagle_build_tilemap_packed(seq_lens: Sequence[int], K: int, depth_count: Optional[Sequence[int]] = None,
                                seg_bounds: Optional[Sequence[int]] = None, device: int = 0,
                                assignment: int = ASSIGN_BY_ANCHOR) -> TileMap:
    """Tile map of a packed batch: `seq_lens` anchors per sequence; `depth_count` per global anchor or None (dense)."""
    lib = load_library()
    i32p = C.POINTER(C.c_int32)
    start = np.ascontiguousarray(np.concatenate([[0], np.cumsum(seq_lens)]), dtype=np.int32)
    L = int(start[-1])
    n = None if depth_count is None else np.ascontiguousarray(depth_count, dtype=np.int32)
    if n is not None and len(n) != L:
        raise ValueError("depth_count must have one entry per anchor of the batch")
    b = None if seg_bounds is None else np.ascontiguousarray(seg_bounds, dtype=np.int32)
    out = C.c_void_p()
    rc = lib.peagle_build_tilemap_packed(None if n is None else n.ctypes.data_as(i32p), L, K, start.ctypes.data_as(i32p),
                                         len(start) - 1, None if b is None else b.ctypes.data_as(i32p),
                                         1 if b is None else len(b) - 1, assignment, device, C.byref(out))
    if rc != 0:
        raise PeagleError(rc, "peagle_build_tilemap_packed")
    return TileMap(out.value)


def peagle_workspace_bytes(tm: TileMap, shape: Shape) -> int:
    return int(load_library().peagle_workspace_bytes(tm.handle, shape.c()))


# --------------------------------------------------------------------------- tensor marshalling

def _ptr(t, name: str, dtype, shape):
    """Device pointer of a torch tensor after checking dtype / shape / contiguity."""
    if t is None:
        return None
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if not t.is_cuda:
        raise ValueError(f"{name}: must live on the GPU")
    return C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def peagle_attn_fwd(tm: TileMap, shape: Shape, seg: int, q, k, v, o, lse, stream=None) -> None:
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    T = tm.tokens(shape.L)
    rc = load_library().peagle_attn_fwd(
        tm.handle, shape.c(), seg,
        _ptr(q, "q", bf, (T, shape.Hq, shape.D)), _ptr(k, "k", bf, (T, shape.Hkv, shape.D)),
        _ptr(v, "v", bf, (T, shape.Hkv, shape.D)), _ptr(o, "o", bf, (T, shape.Hq, shape.D)),
        _ptr(lse, "lse", f32, (shape.Hq, T)), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_fwd")


def peagle_attn_bwd(tm: TileMap, shape: Shape, seg: int, q, k, v, o, d_o, lse, dq, dk_acc, dv_acc, accumulate: int,
                    workspace, stream=None) -> None:
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    T = tm.tokens(shape.L)
    qs, ks = (T, shape.Hq, shape.D), (T, shape.Hkv, shape.D)
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace: expected a contiguous uint8 GPU tensor")
    rc = load_library().peagle_attn_bwd(
        tm.handle, shape.c(), seg, _ptr(q, "q", bf, qs), _ptr(k, "k", bf, ks), _ptr(v, "v", bf, ks),
        _ptr(o, "o", bf, qs), _ptr(d_o, "d_o", bf, qs), _ptr(lse, "lse", f32, (shape.Hq, T)),
        _ptr(dq, "dq", bf, qs), _ptr(dk_acc, "dk_acc", f32, ks), _ptr(dv_acc, "dv_acc", f32, ks), int(accumulate),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_bwd")


def peagle_attn_step_partitioned(tm: TileMap, shape: Shape, seg_begin: int, seg_end: int, q, k, v, d_o, o, lse, dq,
                                 dk_acc, dv_acc, dk_bf16, dv_bf16, workspace, stream=None) -> None:
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    T = tm.tokens(shape.L)
    qs, ks = (T, shape.Hq, shape.D), (T, shape.Hkv, shape.D)
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace: expected a contiguous uint8 GPU tensor")
    rc = load_library().peagle_attn_step_partitioned(
        tm.handle, shape.c(), seg_begin, seg_end, _ptr(q, "q", bf, qs), _ptr(k, "k", bf, ks), _ptr(v, "v", bf, ks),
        _ptr(d_o, "d_o", bf, qs), _ptr(o, "o", bf, qs), _ptr(lse, "lse", f32, (shape.Hq, T)),
        _ptr(dq, "dq", bf, qs), _ptr(dk_acc, "dk_acc", f32, ks), _ptr(dv_acc, "dv_acc", f32, ks),
        _ptr(dk_bf16, "dk_bf16", bf, ks), _ptr(dv_bf16, "dv_bf16", bf, ks),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_step_partitioned")


def peagle_attn_step_profiled(tm: TileMap, shape: Shape, seg_begin: int, seg_end: int, q, k, v, d_o, o, lse, dq,
                              dk_acc, dv_acc, workspace, stream=None) -> dict:
    """Same work as peagle_attn_step_partitioned; returns {kind: (ms, launches)} from HIP events."""
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    T = tm.tokens(shape.L)
    qs, ks = (T, shape.Hq, shape.D), (T, shape.Hkv, shape.D)
    prof = _ProfileC()
    rc = load_library().peagle_attn_step_profiled(
        tm.handle, shape.c(), seg_begin, seg_end, _ptr(q, "q", bf, qs), _ptr(k, "k", bf, ks), _ptr(v, "v", bf, ks),
        _ptr(d_o, "d_o", bf, qs), _ptr(o, "o", bf, qs), _ptr(lse, "lse", f32, (shape.Hq, T)),
        _ptr(dq, "dq", bf, qs), _ptr(dk_acc, "dk_acc", f32, ks), _ptr(dv_acc, "dv_acc", f32, ks),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream), C.byref(prof))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_step_profiled")
    return {name: (float(prof.ms[i]), int(prof.launches[i])) for i, name in enumerate(KERNEL_KINDS)}


def peagle_rope_positions(tm: TileMap, L: int) -> int:
    n = int(load_library().peagle_rope_positions(tm.handle, L))
    if n < 0:
        raise PeagleError(-1, "peagle_rope_positions")
    return n


def peagle_rope_position_ids(tm: TileMap, L: int) -> np.ndarray:
    out = np.zeros(tm.tokens(L), dtype=np.int32)
    rc = load_library().peagle_rope_position_ids(tm.handle, L, out.ctypes.data_as(C.POINTER(C.c_int32)))
    if rc != 0:
        raise PeagleError(rc, "peagle_rope_position_ids")
    return out


def peagle_rope_table(base: float, D: int, n_pos: int, table, stream=None) -> None:
    """Fills `table` (fp32 GPU tensor [n_pos, 2, D/2]) with the cosines and sines of every position."""
    import torch
    rc = load_library().peagle_rope_table(float(base), D, n_pos, _ptr(table, "table", torch.float32, (n_pos, 2, D // 2)),
                                          _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_rope_table")


def peagle_rope_rotate(tm: TileMap, shape: Shape, x, rope_table, out, inverse: bool = False, stream=None) -> None:
    import torch
    T = tm.tokens(shape.L)
    H = x.shape[1]
    n_pos = rope_table.shape[0]
    rc = load_library().peagle_rope_rotate(
        tm.handle, shape.c(), _ptr(x, "x", torch.bfloat16, (T, H, shape.D)), H,
        _ptr(rope_table, "rope_table", torch.float32, (n_pos, 2, shape.D // 2)), n_pos, int(inverse),
        _ptr(out, "out", torch.bfloat16, (T, H, shape.D)), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_rope_rotate")


def peagle_rope_workspace_bytes(tm: TileMap, shape: Shape) -> int:
    n = int(load_library().peagle_rope_workspace_bytes(tm.handle, shape.c()))
    if n == 0:
        raise PeagleError(-3, "peagle_rope_workspace_bytes")
    return n


def _rope_step_args(tm, shape, seg_begin, seg_end, q, k, v, d_o, rope_table, o, lse, dq, dk_acc, dv_acc):
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    T = tm.tokens(shape.L)
    qs, ks = (T, shape.Hq, shape.D), (T, shape.Hkv, shape.D)
    n_pos = rope_table.shape[0]
    return [tm.handle, shape.c(), seg_begin, seg_end, _ptr(q, "q", bf, qs), _ptr(k, "k", bf, ks), _ptr(v, "v", bf, ks),
            _ptr(d_o, "d_o", bf, qs), _ptr(rope_table, "rope_table", f32, (n_pos, 2, shape.D // 2)), n_pos,
            _ptr(o, "o", bf, qs), _ptr(lse, "lse", f32, (shape.Hq, T)), _ptr(dq, "dq", bf, qs),
            _ptr(dk_acc, "dk_acc", f32, ks), _ptr(dv_acc, "dv_acc", f32, ks)], ks


def peagle_attn_step_partitioned_rope(tm: TileMap, shape: Shape, seg_begin: int, seg_end: int, q, k, v, d_o, rope_table,
                                      o, lse, dq, dk_acc, dv_acc, dk_bf16, dv_bf16, workspace, stream=None) -> None:
    import torch
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace: expected a contiguous uint8 GPU tensor")
    args, ks = _rope_step_args(tm, shape, seg_begin, seg_end, q, k, v, d_o, rope_table, o, lse, dq, dk_acc, dv_acc)
    rc = load_library().peagle_attn_step_partitioned_rope(
        *args, _ptr(dk_bf16, "dk_bf16", torch.bfloat16, ks), _ptr(dv_bf16, "dv_bf16", torch.bfloat16, ks),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_step_partitioned_rope")


def peagle_attn_step_rope_profiled(tm: TileMap, shape: Shape, seg_begin: int, seg_end: int, q, k, v, d_o, rope_table,
                                   o, lse, dq, dk_acc, dv_acc, workspace, stream=None) -> dict:
    """Same work as peagle_attn_step_partitioned_rope; returns {kind: (ms, launches)} from HIP events."""
    args, _ = _rope_step_args(tm, shape, seg_begin, seg_end, q, k, v, d_o, rope_table, o, lse, dq, dk_acc, dv_acc)
    prof = _ProfileC()
    rc = load_library().peagle_attn_step_rope_profiled(*args, C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                                       _stream_ptr(stream), C.byref(prof))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_step_rope_profiled")
    return {name: (float(prof.ms[i]), int(prof.launches[i])) for i, name in enumerate(KERNEL_KINDS)}


def peagle_rope_shared_workspace_bytes(tm: TileMap, shape: Shape) -> int:
    n = int(load_library().peagle_rope_shared_workspace_bytes(tm.handle, shape.c()))
    if n == 0:
        raise PeagleError(-3, "peagle_rope_shared_workspace_bytes")
    return n


def peagle_attn_step_rope_shared(tm: TileMap, shape: Shape, q, k0, k_shared, v0, v_shared, d_o, rope_table, o, lse, dq,
                                 dk0, dv0, dk_shared, dv_shared, workspace, stream=None) -> None:
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    T = tm.tokens(shape.L)
    qs, k0s, kss = (T, shape.Hq, shape.D), (shape.L, shape.Hkv, shape.D), (shape.Hkv, shape.D)
    n_pos = rope_table.shape[0]
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace: expected a contiguous uint8 GPU tensor")
    rc = load_library().peagle_attn_step_rope_shared(
        tm.handle, shape.c(), _ptr(q, "q", bf, qs), _ptr(k0, "k0", bf, k0s), _ptr(k_shared, "k_shared", bf, kss),
        _ptr(v0, "v0", bf, k0s), _ptr(v_shared, "v_shared", bf, kss), _ptr(d_o, "d_o", bf, qs),
        _ptr(rope_table, "rope_table", f32, (n_pos, 2, shape.D // 2)), n_pos, _ptr(o, "o", bf, qs),
        _ptr(lse, "lse", f32, (shape.Hq, T)), _ptr(dq, "dq", bf, qs), _ptr(dk0, "dk0", f32, k0s),
        _ptr(dv0, "dv0", f32, k0s), _ptr(dk_shared, "dk_shared", f32, kss), _ptr(dv_shared, "dv_shared", f32, kss),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_attn_step_rope_shared")


class DecodeShape:
    """Shape of one inference-side drafting step: C requests, K new positions each, paged KV cache."""

    def __init__(self, C_: int, K: int, Hq: int, Hkv: int, D: int, n_pages: int, max_pages: int,
                 scale: Optional[float] = None):
        self.C, self.K, self.Hq, self.Hkv, self.D, self.n_pages, self.max_pages = C_, K, Hq, Hkv, D, n_pages, max_pages
        self.scale = float(scale) if scale is not None else 1.0 / float(np.sqrt(D))

    def c(self):
        return C.byref(_DecodeShapeC(self.C, self.K, self.Hq, self.Hkv, self.D, self.scale, self.n_pages,
                                     self.max_pages))


def peagle_draft_decode_splits(shape: DecodeShape) -> int:
    return int(load_library().peagle_draft_decode_splits(shape.c()))


def peagle_draft_decode_workspace_bytes(shape: DecodeShape) -> int:
    n = int(load_library().peagle_draft_decode_workspace_bytes(shape.c()))
    if n == 0:
        raise PeagleError(-3, "peagle_draft_decode_workspace_bytes")
    return n


def peagle_draft_decode(shape: DecodeShape, q_new, k_new, v_new, k_pages, v_pages, block_table, ctx_len, o, lse,
                        status, workspace, stream=None) -> None:
    import torch
    bf, f32, i32 = torch.bfloat16, torch.float32, torch.int32
    s = shape
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace: expected a contiguous uint8 GPU tensor")
    pool = (s.n_pages, s.Hkv, 64, s.D)
    rc = load_library().peagle_draft_decode(
        s.c(), _ptr(q_new, "q_new", bf, (s.C, s.K, s.Hq, s.D)), _ptr(k_new, "k_new", bf, (s.C, s.K, s.Hkv, s.D)),
        _ptr(v_new, "v_new", bf, (s.C, s.K, s.Hkv, s.D)), _ptr(k_pages, "k_pages", bf, pool),
        _ptr(v_pages, "v_pages", bf, pool), _ptr(block_table, "block_table", i32, (s.C, s.max_pages)),
        _ptr(ctx_len, "ctx_len", i32, (s.C,)), _ptr(o, "o", bf, (s.C, s.K, s.Hq, s.D)),
        _ptr(lse, "lse", f32, (s.C, s.Hq, s.K)), _ptr(status, "status", i32, (s.C,)),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_draft_decode")


def peagle_draft_decode_static(shape: DecodeShape, q_new, k_new, v_new, k_pages, v_pages, block_table, ctx_len, o, lse,
                               status, stream=None) -> None:
    import torch
    bf, f32, i32 = torch.bfloat16, torch.float32, torch.int32
    s = shape
    pool = (s.n_pages, s.Hkv, 64, s.D)
    rc = load_library().peagle_draft_decode_static(
        s.c(), _ptr(q_new, "q_new", bf, (s.C, s.K, s.Hq, s.D)), _ptr(k_new, "k_new", bf, (s.C, s.K, s.Hkv, s.D)),
        _ptr(v_new, "v_new", bf, (s.C, s.K, s.Hkv, s.D)), _ptr(k_pages, "k_pages", bf, pool),
        _ptr(v_pages, "v_pages", bf, pool), _ptr(block_table, "block_table", i32, (s.C, s.max_pages)),
        _ptr(ctx_len, "ctx_len", i32, (s.C,)), _ptr(o, "o", bf, (s.C, s.K, s.Hq, s.D)),
        _ptr(lse, "lse", f32, (s.C, s.Hq, s.K)), _ptr(status, "status", i32, (s.C,)), _stream_ptr(stream))
    if rc != 0:
        raise PeagleError(rc, "peagle_draft_decode_static")


def peagle_measure_mfma_ceiling(stream=None, random_operands: bool = False) -> float:
    out = C.c_float(0.0)
    lib = load_library()
    fn = lib.peagle_measure_mfma_ceiling_random if random_operands else lib.peagle_measure_mfma_ceiling
    rc = fn(_stream_ptr(stream), C.byref(out))
    if rc != 0:
        raise PeagleError(rc, "peagle_measure_mfma_ceiling")
    return float(out.value)


def peagle_device_info() -> dict:
    cus, khz = C.c_int32(0), C.c_int32(0)
    rc = load_library().peagle_device_info(C.byref(cus), C.byref(khz))
    if rc != 0:
        raise PeagleError(rc, "peagle_device_info")
    return {"compute_units": int(cus.value), "clock_khz": int(khz.value)}
