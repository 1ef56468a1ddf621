"""Host-side checks of the C ABI: the library loads, exports every declared
entry point, and rejects bad descriptors without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2211_10526_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in os.listdir(inc):
        if f.endswith(".h"):
            text = open(os.path.join(inc, f)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(castling_attn_\w+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = b.lib()
    decl = declared_symbols()
    assert decl == set(b.EXPORTS)
    for name in decl:
        assert hasattr(L, name), name


def good():
    return b.make_desc(2, 4, 196, 64, 14, 14, 3, "bf16")


def test_validate_accepts_benchmark_workloads():
    from paper_2211_10526_amd import inputs
    for wl in inputs.WORKLOADS:
        d = b.make_desc(wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype)
        assert b.validate(d) == b.OK, wl.name


@pytest.mark.parametrize("field,value,status", [
    ("B", 0, b.ERR_INVALID_ARG), ("heads", -1, b.ERR_INVALID_ARG), ("N", 195, b.ERR_INVALID_ARG),
    ("grid_w", 13, b.ERR_INVALID_ARG), ("dw_kernel", 4, b.ERR_INVALID_ARG),
    ("dw_kernel", 0, b.ERR_INVALID_ARG), ("dw_kernel", 11, b.ERR_UNSUPPORTED),
    ("d", 48, b.ERR_UNSUPPORTED), ("d", 0, b.ERR_INVALID_ARG), ("io_dtype", 7, b.ERR_UNSUPPORTED),
    ("norm", 2, b.ERR_INVALID_ARG), ("branches", 8, b.ERR_INVALID_ARG),
    ("eps", -1.0, b.ERR_INVALID_ARG), ("eps", float("nan"), b.ERR_INVALID_ARG),
])
def test_validate_rejects(field, value, status):
    d = good()
    setattr(d, field, value)
    assert b.validate(d) == status


def test_validate_null_and_strerror():
    L = b.lib()
    assert L.castling_attn_validate(None) == b.ERR_INVALID_ARG
    assert b.strerror(b.OK) == "ok"
    for s in (1, 2, 3, 4, 99):
        assert isinstance(b.strerror(s), str) and b.strerror(s)
    # create refuses a bad descriptor before it allocates anything
    h = C.c_void_p(123)
    d = good()
    d.N = 7
    assert L.castling_attn_create(C.byref(d), C.byref(h)) == b.ERR_INVALID_ARG
    assert not h.value
    assert L.castling_attn_create(C.byref(good()), None) == b.ERR_INVALID_ARG
    assert L.castling_attn_destroy(None) == b.OK
    assert L.castling_attn_workspace_bytes(None) == 0
    assert L.castling_attn_num_splits(None) == 0
    assert L.castling_attn_forward(None, None, None, None, None, None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_reduce(None, None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_apply(None, None, None, None, None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_prepare_weights(None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_get_state(None, None, 0, None) == b.ERR_INVALID_ARG
