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
    ("d", 20, b.ERR_UNSUPPORTED), ("d", 136, b.ERR_UNSUPPORTED), ("d", 256, b.ERR_UNSUPPORTED),
    ("d", 0, b.ERR_INVALID_ARG),
    ("io_dtype", 7, b.ERR_UNSUPPORTED),
    ("norm", 2, b.ERR_INVALID_ARG), ("branches", 8, b.ERR_INVALID_ARG),
    ("eps", -1.0, b.ERR_INVALID_ARG), ("eps", float("nan"), b.ERR_INVALID_ARG),
    ("flags", 32, b.ERR_INVALID_ARG),
    ("eps", 1e-39, b.ERR_INVALID_ARG),
])
def test_validate_rejects(field, value, status):
    d = good()
    setattr(d, field, value)
    assert b.validate(d) == status


@pytest.mark.parametrize("d", [8, 16, 24, 48, 64, 96, 120, 128])
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_validate_accepts_head_widths_in_steps_of_eight(d, dtype):
    assert b.validate(b.make_desc(2, 4, 196, d, 14, 14, 3, dtype)) == b.OK


def test_validate_strides():
    B, H, N, d = 2, 4, 196, 64
    fused = b.fused_qkv_strides(H, N, d)
    tok = b.token_major_strides(H, N, d)
    mk = lambda ins, outs: b.make_desc(B, H, N, d, 14, 14, 3, "bf16", in_strides=ins, out_strides=outs)
    assert b.validate(mk(fused, tok)) == b.OK
    assert b.validate(mk(fused, None)) == b.OK
    assert b.validate(mk(None, tok)) == b.OK
    assert b.validate(mk((H * N * d, N * d, d), (H * N * d, N * d, d))) == b.OK
    # not a multiple of 16 bytes, negative, partly zero, token stride below d
    assert b.validate(mk((fused[0], fused[1], fused[2] + 4), None)) == b.ERR_INVALID_ARG
    assert b.validate(mk((fused[0], -64, fused[2]), None)) == b.ERR_INVALID_ARG
    assert b.validate(mk((0, fused[1], fused[2]), None)) == b.ERR_INVALID_ARG
    assert b.validate(mk(None, (tok[0], tok[1], 32))) == b.ERR_INVALID_ARG
    # fp32 rows need 4-element multiples only
    f = b.make_desc(B, H, N, 32, 14, 14, 3, "f32", in_strides=(N * 3 * H * 36, 36, 3 * H * 36))
    assert b.validate(f) == b.OK
    # one unit's tokens must stay inside 32-bit byte offsets
    big = b.make_desc(1, 1, 16384, 64, 128, 128, 3, "bf16", in_strides=(1 << 34, 64, 1 << 18))
    assert b.validate(big) == b.ERR_UNSUPPORTED
    # ... with the contiguous default strides as well: 2^25 tokens of 64 bf16 = 4 GiB per unit
    assert b.validate(b.make_desc(1, 1, 1 << 25, 64, 4096, 8192, 3, "bf16")) == b.ERR_UNSUPPORTED
    assert b.validate(b.make_desc(1, 1, 1 << 24, 64, 4096, 4096, 3, "bf16")) == b.OK
    # pass 2 counts 4 x 16 pieces of the grid in 32 bits: 65535 units of a 262144 x 1 grid
    assert b.validate(b.make_desc(255, 257, 1 << 18, 16, 1 << 18, 1, 3, "bf16")) == b.ERR_UNSUPPORTED


def test_validate_downsampling_fields():
    mk = lambda **kw: b.make_desc(2, 4, 196, 64, 14, 14, 3, "bf16", **kw)
    assert C.sizeof(b.Desc) == 136
    assert b.validate(mk(q_pool=1)) == b.OK
    assert b.validate(mk(q_pool=2, flags=b.FLAG_RESIDUAL_Q)) == b.OK
    assert b.validate(mk(q_pool=2, q_strides=(49 * 4 * 72, 72, 4 * 72))) == b.OK
    assert b.validate(mk(q_pool=3)) == b.ERR_UNSUPPORTED
    assert b.validate(mk(q_pool=-1)) == b.ERR_INVALID_ARG
    # pooled queries and class tokens together are not covered
    assert b.validate(b.make_desc(2, 4, 197, 64, 14, 14, 3, "bf16", extra_tokens=1, q_pool=2)) \
        == b.ERR_UNSUPPORTED
    # q has strides of its own only where it is pooled; they follow the rules of the others
    assert b.validate(mk(q_strides=(49 * 4 * 64, 64, 4 * 64))) == b.ERR_INVALID_ARG
    assert b.validate(mk(q_pool=2, q_strides=(49 * 4 * 64, 60, 4 * 64))) == b.ERR_INVALID_ARG
    assert b.validate(mk(q_pool=2, q_strides=(49 * 4 * 64, 64, 32))) == b.ERR_INVALID_ARG
    # the residual query belongs to the attention branch
    assert b.validate(mk(flags=b.FLAG_RESIDUAL_Q, branches=b.BRANCH_DWCONV)) == b.ERR_INVALID_ARG
    assert b.validate(mk(flags=b.FLAG_RESIDUAL_Q, branches=b.BRANCH_LINEAR)) == b.OK
    assert b.validate(mk(flags=b.FLAG_TRAINING)) == b.OK
    assert b.validate(mk(flags=32)) == b.ERR_INVALID_ARG
    assert b.validate(mk(flags=b.FLAG_SEPARATE_PASSES | b.FLAG_VECTOR_ALU)) == b.OK
    d = mk()
    d.reserved0 = 1
    assert b.validate(d) == b.ERR_INVALID_ARG


def test_validate_null_and_strerror():
    L = b.lib()
    assert L.castling_attn_validate(None) == b.ERR_INVALID_ARG
    assert b.strerror(b.OK) == "ok"
    for s in (1, 2, 3, 4, 5, 99):
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
    assert L.castling_attn_num_launches(None) == 0
    assert L.castling_attn_pairwise(None, None, None, None, None, None, None, None) == b.ERR_INVALID_ARG
    assert C.sizeof(b.PairParams) == 20  # mode, normalize, scale, threshold, accumulate
    assert L.castling_attn_forward(None, None, None, None, None, None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_reduce(None, None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_apply(None, None, None, None, None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_prepare_weights(None, None, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_get_state(None, None, 0, None) == b.ERR_INVALID_ARG
    assert L.castling_attn_backward(*([None] * 12)) == b.ERR_INVALID_ARG
    # the forward without allocation checks its descriptor before it touches the device
    assert L.castling_attn_forward_static(None, *([None] * 7)) == b.ERR_INVALID_ARG
    assert L.castling_attn_forward_static(C.byref(d), *([None] * 7)) == b.ERR_INVALID_ARG
    t = good()
    t.flags = b.FLAG_TRAINING
    assert L.castling_attn_forward_static(C.byref(t), *([None] * 7)) == b.ERR_INVALID_ARG
    assert "scratch" in b.strerror(b.ERR_TOO_LARGE) and b.ERR_TOO_LARGE == 5
    import os
    import re
    header = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include",
                               "castling_attn.h")).read()
    m = re.search(r"#define CASTLING_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert m and b.STATIC_SCRATCH_BYTES == int(m.group(1)) << int(m.group(2))
