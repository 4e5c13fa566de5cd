"""ctypes binding of the C ABI in include/mmm.h.

Argument marshalling only: every step of the path runs in the HIP library.
PyTorch tensors are used as device buffers and for the stream handle.  There is
no fallback: if the library is not built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

# PyTorch ships its own HIP runtime (same soname as the system one).  Device
# pointers and streams handed to the library come from PyTorch, so its runtime
# must be the one already loaded when libmmm_hip.so is opened; loading ours first
# leaves the process with a runtime that reports no device.
import torch  # noqa: F401  (must precede ctypes.CDLL below)

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libmmm_hip.so")

MMM_OK = 0
MMM_ERR_INVALID_ARG, MMM_ERR_SHAPE, MMM_ERR_DTYPE, MMM_ERR_WORKSPACE, MMM_ERR_MAPS_MISMATCH, MMM_ERR_DEVICE = range(1, 7)
MMM_F32, MMM_BF16, MMM_F16, MMM_F64 = 0, 1, 2, 3
MMM_PRED_NONZERO, MMM_PRED_GT, MMM_PRED_ABS_GT = 0, 1, 2
MMM_PATH_AUTO, MMM_PATH_MATRIX, MMM_PATH_PAIRS = -1, 0, 1

EXPORTS = [
    "mmm_maps_workspace_bytes", "mmm_maps_init", "mmm_maps_release", "mmm_build_maps", "mmm_maps_view",
    "mmm_maps_view_derived", "mmm_maps_view_compacted", "mmm_maps_view_lists", "mmm_debug_k_lists", "mmm_maps_stats", "mmm_matmul", "mmm_matmul_static_scratch", "mmm_matmul_fused",
    "mmm_maps_set_path", "mmm_matmul_path", "mmm_set_option", "mmm_matmul_variant_count",
    "mmm_matmul_variant_name", "mmm_matmul_plan", "mmm_maps_set_plan", "mmm_status_string", "mmm_last_device_error",
]


class MaskA(ctypes.Structure):
    _fields_ = [("pred", ctypes.c_int32), ("threshold", ctypes.c_float), ("keep_bits", ctypes.c_void_p)]


class MaskB(ctypes.Structure):
    _fields_ = [("block_width", ctypes.c_int32), ("keep_rows", ctypes.c_void_p), ("keep_blocks", ctypes.c_void_p)]


class MmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = ""
        if status == MMM_ERR_DEVICE or (status == MMM_ERR_WORKSPACE and where == "mmm_matmul_static_scratch"):
            detail = f" [{mmm_last_device_error()}]"
        super().__init__(f"{where}: {status_string(status)} (status {status}){detail}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    i64, i32, vp = c.c_int64, c.c_int32, c.c_void_p
    lib.mmm_maps_workspace_bytes.argtypes = [i64, i64, i64, i32, c.POINTER(c.c_size_t)]
    lib.mmm_maps_init.argtypes = [vp, c.c_size_t, i64, i64, i64, i32, c.POINTER(vp)]
    lib.mmm_maps_release.argtypes = [vp]
    lib.mmm_maps_release.restype = None
    lib.mmm_build_maps.argtypes = [vp, i32, vp, i64, c.POINTER(MaskA), vp, i64, c.POINTER(MaskB), vp]
    lib.mmm_maps_view.argtypes = [vp, c.POINTER(vp), c.POINTER(i64), c.POINTER(vp), c.POINTER(i64)]
    lib.mmm_maps_view_derived.argtypes = [vp, c.POINTER(vp), c.POINTER(vp), c.POINTER(i64)]
    lib.mmm_maps_view_compacted.argtypes = [vp, c.POINTER(i32), c.POINTER(vp), c.POINTER(vp), c.POINTER(vp), c.POINTER(vp)]
    lib.mmm_debug_k_lists.argtypes = [vp, vp, c.c_size_t, c.POINTER(c.c_size_t), vp]
    lib.mmm_maps_view_lists.argtypes = [vp, c.POINTER(vp), c.POINTER(vp), c.POINTER(i64), c.POINTER(i64), c.POINTER(i64)]
    lib.mmm_maps_stats.argtypes = [vp, c.POINTER(c.c_uint64), c.POINTER(c.c_uint64), c.POINTER(c.c_uint64), vp]
    lib.mmm_matmul.argtypes = [vp, i32, vp, i64, vp, i64, vp, i64, i32, vp]
    lib.mmm_matmul_static_scratch.argtypes = [vp, i32, vp, i64, vp, i64, vp, i64, i32, vp]
    lib.mmm_matmul_fused.argtypes = [vp, i32, vp, i64, c.POINTER(MaskA), vp, i64, vp, i64, i32, vp]
    lib.mmm_maps_set_path.argtypes = [vp, i32]
    lib.mmm_matmul_path.argtypes = [vp, c.POINTER(i32)]
    lib.mmm_set_option.argtypes = [c.c_char_p, i64]
    lib.mmm_maps_set_plan.argtypes = [vp, i32, i32]
    lib.mmm_matmul_variant_count.restype = i32
    lib.mmm_matmul_variant_name.argtypes = [i32]
    lib.mmm_matmul_variant_name.restype = c.c_char_p
    lib.mmm_matmul_plan.argtypes = [vp, i32, c.POINTER(i32), c.POINTER(i32), c.POINTER(i64)]
    lib.mmm_status_string.argtypes = [i32]
    lib.mmm_status_string.restype = c.c_char_p
    lib.mmm_last_device_error.restype = c.c_char_p
    return lib


lib = _load()


def status_string(st: int) -> str:
    return lib.mmm_status_string(int(st)).decode()


def mmm_last_device_error() -> str:
    return lib.mmm_last_device_error().decode()


def _check(st: int, where: str) -> None:
    if st != MMM_OK:
        raise MmmError(st, where)


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or pass an int / None through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def mmm_maps_workspace_bytes(M: int, K: int, N: int, block_width: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib.mmm_maps_workspace_bytes(M, K, N, block_width, ctypes.byref(out)), "mmm_maps_workspace_bytes")
    return out.value


def mmm_maps_init(dev_workspace, workspace_bytes: int, M: int, K: int, N: int, block_width: int) -> int:
    out = ctypes.c_void_p(None)
    _check(lib.mmm_maps_init(_ptr(dev_workspace), workspace_bytes, M, K, N, block_width, ctypes.byref(out)),
           "mmm_maps_init")
    return out.value


def mmm_maps_release(maps: Optional[int]) -> None:
    lib.mmm_maps_release(maps)


def mmm_build_maps(maps: int, dt: int, X, ldx: int, ma: Optional[MaskA], Y, ldy: int, mb: Optional[MaskB],
                   stream=None) -> None:
    _check(lib.mmm_build_maps(maps, dt, _ptr(X), ldx, ctypes.byref(ma) if ma is not None else None,
                              _ptr(Y), ldy, ctypes.byref(mb) if mb is not None else None, _stream(stream)),
           "mmm_build_maps")


def mmm_maps_view(maps: int):
    """(a_bits address, a_row_words, b_bits address, b_row_words)"""
    a, b = ctypes.c_void_p(None), ctypes.c_void_p(None)
    aw, bw = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib.mmm_maps_view(maps, ctypes.byref(a), ctypes.byref(aw), ctypes.byref(b), ctypes.byref(bw)),
           "mmm_maps_view")
    return a.value, aw.value, b.value, bw.value


def mmm_maps_view_derived(maps: int):
    """(a_colany address, bt_bits address, k_words)"""
    a, b = ctypes.c_void_p(None), ctypes.c_void_p(None)
    kw = ctypes.c_int64(0)
    _check(lib.mmm_maps_view_derived(maps, ctypes.byref(a), ctypes.byref(b), ctypes.byref(kw)), "mmm_maps_view_derived")
    return a.value, b.value, kw.value


def mmm_maps_view_compacted(maps: int):
    """(on, live_count address, kmap address, a_colany_c address, btc_bits address)"""
    on = ctypes.c_int32(0)
    a, b, c_, d = (ctypes.c_void_p(None) for _ in range(4))
    _check(lib.mmm_maps_view_compacted(maps, ctypes.byref(on), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c_),
                                       ctypes.byref(d)), "mmm_maps_view_compacted")
    return bool(on.value), a.value, b.value, c_.value, d.value


def mmm_debug_k_lists(maps: int, out=None, out_bytes: int = 0, stream=None) -> int:
    """Writes the matrix kernel's k lists to `out` (device memory); returns the bytes needed (out=None: only that)."""
    need = ctypes.c_size_t(0)
    _check(lib.mmm_debug_k_lists(maps, _ptr(out), out_bytes, ctypes.byref(need), _stream(stream)), "mmm_debug_k_lists")
    return need.value


def mmm_maps_view_lists(maps: int):
    """(counts address, entries address, blocks_m, blocks_k, capacity)"""
    a, b = ctypes.c_void_p(None), ctypes.c_void_p(None)
    bm, bk, cap = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib.mmm_maps_view_lists(maps, ctypes.byref(a), ctypes.byref(b), ctypes.byref(bm), ctypes.byref(bk),
                                   ctypes.byref(cap)), "mmm_maps_view_lists")
    return a.value, b.value, bm.value, bk.value, cap.value


def mmm_maps_stats(maps: int, stream=None):
    """(nnz_a, occupied_blocks_b, useful_macs); waits for the stream."""
    a, b, m = ctypes.c_uint64(0), ctypes.c_uint64(0), ctypes.c_uint64(0)
    _check(lib.mmm_maps_stats(maps, ctypes.byref(a), ctypes.byref(b), ctypes.byref(m), _stream(stream)), "mmm_maps_stats")
    return a.value, b.value, m.value


def mmm_matmul(maps: int, dt: int, X, ldx: int, Y, ldy: int, C, ldc: int, accumulate: int = 0, stream=None) -> None:
    _check(lib.mmm_matmul(maps, dt, _ptr(X), ldx, _ptr(Y), ldy, _ptr(C), ldc, int(accumulate), _stream(stream)),
           "mmm_matmul")


def mmm_matmul_static_scratch(maps: int, dt: int, X, ldx: int, Y, ldy: int, C, ldc: int, accumulate: int = 0,
                              stream=None) -> None:
    _check(lib.mmm_matmul_static_scratch(maps, dt, _ptr(X), ldx, _ptr(Y), ldy, _ptr(C), ldc, int(accumulate),
                                         _stream(stream)), "mmm_matmul_static_scratch")


def mmm_matmul_fused(maps: int, dt: int, X, ldx: int, ma: MaskA, Y, ldy: int, C, ldc: int, accumulate: int = 0,
                     stream=None) -> None:
    _check(lib.mmm_matmul_fused(maps, dt, _ptr(X), ldx, ctypes.byref(ma), _ptr(Y), ldy, _ptr(C), ldc, int(accumulate),
                                _stream(stream)), "mmm_matmul_fused")


def mmm_maps_set_path(maps: int, path: int = -1) -> None:
    _check(lib.mmm_maps_set_path(maps, int(path)), "mmm_maps_set_path")


def mmm_matmul_path(maps: int) -> int:
    v = ctypes.c_int32(0)
    _check(lib.mmm_matmul_path(maps, ctypes.byref(v)), "mmm_matmul_path")
    return v.value


def mmm_maps_set_plan(maps: int, variant: int = -1, split_k: int = 0) -> None:
    _check(lib.mmm_maps_set_plan(maps, int(variant), int(split_k)), "mmm_maps_set_plan")


def mmm_set_option(name: str, value: int) -> None:
    _check(lib.mmm_set_option(name.encode(), int(value)), f"mmm_set_option({name})")


def mmm_matmul_variant_count() -> int:
    return int(lib.mmm_matmul_variant_count())


def mmm_matmul_variant_name(i: int) -> Optional[str]:
    s = lib.mmm_matmul_variant_name(i)
    return None if s is None else s.decode()


def mmm_matmul_plan(maps: int, dt: int):
    """(variant, split_k, workgroups)"""
    v, s, w = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int64(0)
    _check(lib.mmm_matmul_plan(maps, dt, ctypes.byref(v), ctypes.byref(s), ctypes.byref(w)), "mmm_matmul_plan")
    return v.value, s.value, w.value
