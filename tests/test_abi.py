"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device.  No GPU
needed: every call below returns from validation."""
import ctypes
import os
import re

import pytest

from paper_2405_03133_amd import binding as lb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # aligned, non-NULL, never dereferenced on these paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lory.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lory_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(lb.EXPORTS) == set(names)
    L = lb.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings():
    assert re.match(r"^\d+\.\d+$", lb.version())
    seen = {lb.status_string(i) for i in range(0, 7)}
    assert len(seen) == 7
    assert lb.status_string(99) == "unknown status"


def shape(**kw):
    base = dict(B=2, L=512, T=128, d=64, d_ff=256, E=4, dtype=lb.LORY_F32)
    base.update(kw)
    return lb.make_shape(**base)


@pytest.mark.parametrize("kw", [dict(B=0), dict(L=-1), dict(T=0), dict(d=0), dict(d_ff=0), dict(E=0),
                                dict(L=500), dict(E=65),
                                dict(dtype=lb.LORY_BF16, d=96), dict(dtype=lb.LORY_BF16, d_ff=200),
                                dict(dtype=lb.LORY_BF16, T=32, L=512)])
def test_bad_shapes_are_rejected(kw):
    out = ctypes.c_size_t(123)
    rc = lb.lib().lory_workspace_bytes(ctypes.byref(shape(**kw)), lb.LORY_PASS_FWD, ctypes.byref(out))
    assert rc == lb.LORY_ERR_SHAPE
    assert out.value == 123


def test_bad_dtype_and_nulls():
    L = lb.lib()
    out = ctypes.c_size_t(0)
    assert L.lory_workspace_bytes(ctypes.byref(shape(dtype=7)), 0, ctypes.byref(out)) == lb.LORY_ERR_DTYPE
    assert L.lory_workspace_bytes(None, 0, ctypes.byref(out)) == lb.LORY_ERR_NULL
    assert L.lory_workspace_bytes(ctypes.byref(shape()), 0, None) == lb.LORY_ERR_NULL
    assert L.lory_workspace_bytes(ctypes.byref(shape()), 5, ctypes.byref(out)) == lb.LORY_ERR_SHAPE
    s = shape()
    assert L.lory_route(ctypes.byref(s), None, FAKE, FAKE, None, None) == lb.LORY_ERR_NULL
    assert L.lory_route(ctypes.byref(s), FAKE, FAKE, None, None, None) == lb.LORY_ERR_NULL
    assert L.lory_route(ctypes.byref(s), FAKE + 4, FAKE, FAKE, None, None) == lb.LORY_ERR_ALIGN
    assert L.lory_route(ctypes.byref(shape(L=500)), FAKE, FAKE, FAKE, None, None) == lb.LORY_ERR_SHAPE


def test_route_bwd_validation():
    L = lb.lib()
    s = shape()
    sp = ctypes.byref(s)
    F = FAKE
    for i in range(6):
        args = [F] * 6
        args[i] = None
        assert L.lory_route_bwd(sp, *args, 0, None) == lb.LORY_ERR_NULL
        args[i] = F + 4
        assert L.lory_route_bwd(sp, *args, 0, None) == lb.LORY_ERR_ALIGN
    assert L.lory_route_bwd(sp, F, F, F, F, F, F, 2, None) == lb.LORY_ERR_SHAPE
    assert L.lory_route_bwd(ctypes.byref(shape(L=500)), F, F, F, F, F, F, 0, None) == lb.LORY_ERR_SHAPE
    assert L.lory_route_bwd(None, F, F, F, F, F, F, 0, None) == lb.LORY_ERR_NULL


def test_inference_entry_points_validation():
    L = lb.lib()
    F = FAKE
    s = shape(L=37, T=37)                      # any prompt length, one segment per sequence
    sp = ctypes.byref(s)
    need = lb.lory_workspace_bytes(s, lb.LORY_PASS_DENSE)
    assert need > 0 and need % 256 == 0
    bad = ctypes.byref(shape(L=64, T=32))      # T != L
    out = ctypes.c_size_t(5)
    assert L.lory_workspace_bytes(bad, lb.LORY_PASS_DENSE, ctypes.byref(out)) == lb.LORY_ERR_SHAPE
    assert out.value == 5
    assert L.lory_prompt_merge(bad, F, None, F, F, F, F, F, F, None) == lb.LORY_ERR_SHAPE
    assert L.lory_dense_ffn_fwd(bad, F, F, F, F, need, None) == lb.LORY_ERR_SHAPE
    for i in range(8):
        if i == 1:
            continue                           # prompt_len_opt may be NULL
        args = [F] * 8
        args[i] = None
        assert L.lory_prompt_merge(sp, *args, None) == lb.LORY_ERR_NULL
        args[i] = F + 8
        assert L.lory_prompt_merge(sp, *args, None) == lb.LORY_ERR_ALIGN
    args = [F] * 8
    args[1] = F + 2                            # lengths need 4-byte alignment only
    assert L.lory_prompt_merge(sp, *args, None) == lb.LORY_ERR_ALIGN
    for i in range(4):
        args = [F] * 4
        args[i] = None
        assert L.lory_dense_ffn_fwd(sp, *args, need, None) == lb.LORY_ERR_NULL
        args[i] = F + 8
        assert L.lory_dense_ffn_fwd(sp, *args, need, None) == lb.LORY_ERR_ALIGN
    assert L.lory_dense_ffn_fwd(sp, F, F, F, F, need - 1, None) == lb.LORY_ERR_WORKSPACE
    # bf16: d and d_ff granularity still applies, the token count does not
    assert lb.lory_workspace_bytes(shape(dtype=lb.LORY_BF16, L=5, T=5, d=64, d_ff=128), lb.LORY_PASS_DENSE) > 0
    assert L.lory_workspace_bytes(ctypes.byref(shape(dtype=lb.LORY_BF16, L=5, T=5, d=72)), lb.LORY_PASS_DENSE,
                                  ctypes.byref(out)) == lb.LORY_ERR_SHAPE


@pytest.mark.parametrize("dtype", [lb.LORY_F32, lb.LORY_BF16])
def test_workspace_query_and_ffn_validation(dtype):
    L = lb.lib()
    s = shape(dtype=dtype, T=128, d=64, d_ff=256)
    need_f = lb.lory_workspace_bytes(s, lb.LORY_PASS_FWD)
    need_b = lb.lory_workspace_bytes(s, lb.LORY_PASS_BWD)
    assert need_f > 0 and need_b > 0 and need_f % 256 == 0 and need_b % 256 == 0
    sp = ctypes.byref(s)
    F = FAKE
    # forward: NULL, mismatched save pair, alignment, short workspace
    assert L.lory_merged_ffn_fwd(sp, None, F, F, F, F, F, None, None, None, F, need_f, None) == lb.LORY_ERR_NULL
    assert L.lory_merged_ffn_fwd(sp, F, F, F, F, F, F, F, None, None, F, need_f, None) == lb.LORY_ERR_NULL
    assert L.lory_merged_ffn_fwd(sp, F, F, F, F + 8, F, F, None, None, None, F, need_f, None) == lb.LORY_ERR_ALIGN
    assert L.lory_merged_ffn_fwd(sp, F, F, F, F, F, F, None, None, None, F, need_f - 1, None) == lb.LORY_ERR_WORKSPACE
    save = lb.lory_merged_save_bytes(s)
    if dtype == lb.LORY_F32:
        assert save == 0
        assert L.lory_merged_ffn_fwd(sp, F, F, F, F, F, F, None, None, F, F, need_f, None) == lb.LORY_ERR_SHAPE
    else:
        assert save == 3 * 8 * 64 * 256 * 2
    # backward
    args = [F] * 8 + [None] + [F] * 4   # ..., U_save, Wbar_save = NULL, dX, dWg, dWu, dWd
    assert L.lory_merged_ffn_bwd(sp, *args, lb.LORY_F32, 0, None, F, need_b, None) == lb.LORY_ERR_NULL
    assert L.lory_merged_ffn_bwd(sp, *args, 9, 0, F, F, need_b, None) == lb.LORY_ERR_DTYPE
    assert L.lory_merged_ffn_bwd(sp, *args, lb.LORY_F32, 2, F, F, need_b, None) == lb.LORY_ERR_SHAPE
    assert L.lory_merged_ffn_bwd(sp, *args, lb.LORY_F32, 0, F, F, need_b - 1, None) == lb.LORY_ERR_WORKSPACE
    if dtype == lb.LORY_F32:
        assert L.lory_merged_ffn_bwd(sp, *args, lb.LORY_BF16, 0, F, F, need_b, None) == lb.LORY_ERR_DTYPE
    bad = list(args)
    bad[10] = F + 2
    assert L.lory_merged_ffn_bwd(sp, *bad, lb.LORY_F32, 0, F, F, need_b, None) == lb.LORY_ERR_ALIGN
