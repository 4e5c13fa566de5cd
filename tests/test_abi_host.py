"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every declared symbol, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2402_14118_amd as mm
from paper_2402_14118_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = declared_symbols()
    assert len(syms) >= 13
    for s in syms:
        assert hasattr(B.lib, s), s
    assert set(syms) == set(B.EXPORTS)


def test_status_strings():
    assert B.status_string(0) == "ok"
    assert len({B.status_string(i) for i in range(7)}) == 7


def test_workspace_bytes_and_shape_errors():
    n = mm.mmm_maps_workspace_bytes(2048, 2048, 2048, 16)
    maps_only = 2048 * 32 * 8 + 64 * 32 * 8 + 2048 * 2 * 8 + 128 * 32 * 8
    assert n >= maps_only and n % 256 == 0
    for bad in [(0, 8, 8, 8), (8, 0, 8, 8), (8, 8, 0, 8), (8, 8, 12, 8), (8, 8, 16, 4), (8, 8, 64, 64), (-1, 8, 8, 8)]:
        with pytest.raises(mm.MmmError) as e:
            mm.mmm_maps_workspace_bytes(*bad)
        assert e.value.status == B.MMM_ERR_SHAPE
    assert B.lib.mmm_maps_workspace_bytes(8, 8, 8, 8, None) == B.MMM_ERR_INVALID_ARG


def test_init_and_call_validation_without_device():
    need = mm.mmm_maps_workspace_bytes(64, 128, 64, 16)
    fake = 0x7000_0000_0000          # never dereferenced on the host
    out = ctypes.c_void_p(None)
    assert B.lib.mmm_maps_init(None, need, 64, 128, 64, 16, ctypes.byref(out)) == B.MMM_ERR_WORKSPACE
    assert B.lib.mmm_maps_init(fake + 8, need, 64, 128, 64, 16, ctypes.byref(out)) == B.MMM_ERR_WORKSPACE
    assert B.lib.mmm_maps_init(fake, need - 1, 64, 128, 64, 16, ctypes.byref(out)) == B.MMM_ERR_WORKSPACE
    assert B.lib.mmm_maps_init(fake, need, 64, 128, 60, 16, ctypes.byref(out)) == B.MMM_ERR_SHAPE
    assert B.lib.mmm_maps_init(fake, need, 64, 128, 64, 16, None) == B.MMM_ERR_INVALID_ARG
    assert out.value is None
    maps = mm.mmm_maps_init(fake, need, 64, 128, 64, 16)
    try:
        ma, mb = mm.MaskA(0, 0.0, None), mm.MaskB(16, None, None)
        X = Y = C = fake + 4096
        L = B.lib
        r = ctypes.byref
        assert L.mmm_build_maps(None, 0, X, 128, r(ma), Y, 64, r(mb), None) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_build_maps(maps, 0, None, 128, r(ma), None, 64, r(mb), None) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_build_maps(maps, 0, X, 128, None, Y, 64, r(mb), None) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_build_maps(maps, 7, X, 128, r(ma), Y, 64, r(mb), None) == B.MMM_ERR_DTYPE
        assert L.mmm_build_maps(maps, 0, X, 127, r(ma), Y, 64, r(mb), None) == B.MMM_ERR_SHAPE
        assert L.mmm_build_maps(maps, 0, X, 128, r(ma), Y, 63, r(mb), None) == B.MMM_ERR_SHAPE
        assert L.mmm_build_maps(maps, 0, X + 2, 128, r(ma), Y, 64, r(mb), None) == B.MMM_ERR_DTYPE
        # leading dimensions of 2^22 elements and more are refused by the builder and by the multiplication alike
        big = 1 << 22
        assert L.mmm_build_maps(maps, 0, X, big, r(ma), Y, 64, r(mb), None) == B.MMM_ERR_SHAPE
        assert L.mmm_build_maps(maps, 0, X, 128, r(ma), Y, big, r(mb), None) == B.MMM_ERR_SHAPE
        assert L.mmm_build_maps(maps, 0, None, 0, None, Y, big, r(mb), None) == B.MMM_ERR_SHAPE
        assert L.mmm_matmul(maps, 0, X, big, Y, 64, C, 64, 0, None) == B.MMM_ERR_SHAPE
        assert L.mmm_matmul(maps, 0, X, 128, Y, big, C, 64, 0, None) == B.MMM_ERR_SHAPE
        assert L.mmm_build_maps(maps, 0, X, 128, r(mm.MaskA(3, 0.0, None)), Y, 64, r(mb), None) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_build_maps(maps, 0, X, 128, r(ma), Y, 64, r(mm.MaskB(8, None, None)), None) == B.MMM_ERR_SHAPE
        # nothing built yet: the multiplication and the statistics refuse
        assert L.mmm_matmul(maps, 0, X, 128, Y, 64, C, 64, 0, None) == B.MMM_ERR_MAPS_MISMATCH
        assert L.mmm_maps_stats(maps, None, None, None, None) == B.MMM_ERR_MAPS_MISMATCH
        assert L.mmm_matmul(maps, 0, None, 128, Y, 64, C, 64, 0, None) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_matmul(maps, 0, X, 128, Y, 64, C, 63, 0, None) == B.MMM_ERR_SHAPE
        assert L.mmm_matmul(maps, 4, X, 128, Y, 64, C, 64, 0, None) == B.MMM_ERR_DTYPE      # 3 is MMM_F64
        assert L.mmm_matmul(None, 0, X, 128, Y, 64, C, 64, 0, None) == B.MMM_ERR_INVALID_ARG
        a, aw, b, bw = mm.mmm_maps_view(maps)
        assert a == fake and aw == 2 and bw == 1 and b > a
        ca, bt, kw = mm.mmm_maps_view_derived(maps)
        assert a < ca < b < bt and kw == 2
        v, s, wg = mm.mmm_matmul_plan(maps, 0)
        assert 0 <= v < mm.mmm_matmul_variant_count() and s >= 1 and wg >= 1
        # a plan fixed for the handle wins over the automatic choice; what cannot be used is adjusted
        nv = mm.mmm_matmul_variant_count()
        assert L.mmm_maps_set_plan(maps, nv, 0) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_maps_set_plan(maps, 0, -1) == B.MMM_ERR_INVALID_ARG
        assert L.mmm_maps_set_plan(None, 0, 1) == B.MMM_ERR_INVALID_ARG
        for cand in range(nv):
            mm.mmm_maps_set_plan(maps, cand, 1)
            v2, s2, _ = mm.mmm_matmul_plan(maps, 0)
            short = mm.mmm_matmul_variant_name(cand).startswith("R2")   # 32-row kernels cannot serve M = 64
            assert s2 == 1 and ((v2 == cand) != short)
        mm.mmm_maps_set_plan(maps, 0, 4096)
        assert mm.mmm_matmul_plan(maps, 0)[1] == 1        # K = 128 is a single step: nothing to split
        mm.mmm_maps_set_plan(maps)
        assert mm.mmm_matmul_plan(maps, 0)[:2] == (v, s)
    finally:
        mm.mmm_maps_release(maps)
    mm.mmm_maps_release(None)


def test_options():
    with pytest.raises(mm.MmmError):
        mm.mmm_set_option("no_such_option", 1)
    with pytest.raises(mm.MmmError):
        mm.mmm_set_option("matmul_variant", mm.mmm_matmul_variant_count())
    mm.mmm_set_option("matmul_variant", 0)
    mm.mmm_set_option("matmul_variant", -1)
    mm.mmm_set_option("split_k", 0)
    assert mm.mmm_matmul_variant_name(-1) is None
    assert all(mm.mmm_matmul_variant_name(i) for i in range(mm.mmm_matmul_variant_count()))
