"""GPU parity with class tokens: units of extra + H * W tokens whose first `extra` tokens are
not on the grid.  They take part in the attention sums (state, row sums) and receive the linear
branch; the DWConv term is defined on the grid only."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import STATE_TOL, TOL, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# (grid workload, extra tokens): DeiT-style 14 x 14 + class token (one-kernel path), a
# distillation-token pair, two-pass matrix-core shapes, the vector-ALU kernels, fp16
CASES = [
    (Workload("c_bf16_14x14_k3", "bf16", 2, 3, 64, 14, 14, 3), 1),
    (Workload("c_bf16_14x14_k5", "bf16", 1, 2, 64, 14, 14, 5), 2),
    (Workload("c_bf16_20x24_k3", "bf16", 1, 3, 64, 20, 24, 3), 1),
    (Workload("c_bf16_17x33_k9", "bf16", 2, 1, 64, 17, 33, 9), 2),
    (Workload("c_f16_16x18_k7", "f16", 1, 2, 64, 16, 18, 7), 1),
    (Workload("c_f32_d32_14x14_k3", "f32", 1, 4, 32, 14, 14, 3), 1),
    (Workload("c_bf16_d32_9x11_k5", "bf16", 1, 2, 32, 9, 11, 5), 3),
    (Workload("c_f16_d128_6x7_k3", "f16", 1, 2, 128, 6, 7, 3), 1),
    (Workload("c_bf16_d96_7x7_k3", "bf16", 1, 2, 96, 7, 7, 3), 1),
    (Workload("c_f32_d48_8x8_k5", "f32", 1, 2, 48, 8, 8, 5), 2),
]


def draw(wl, extra, seed):
    """Inputs with extra + N tokens per unit: drawn as a 1 x (extra + N) grid of the same unit
    shape (the filters depend on heads, d and k only)."""
    flat = Workload(wl.name, wl.dtype, wl.B, wl.heads, wl.d, 1, wl.N + extra, wl.dw_kernel)
    return inputs.make_inputs(flat, seed=seed, with_bias=True)


def run(wl, extra, x, norm, branches, want_state=False, fused_layout=False, flags=0):
    dev = torch.device("cuda:0")
    B, H, N, d = wl.B, wl.heads, wl.N + extra, wl.d
    w, bias = x["w"].to(dev), x["bias"].to(dev)
    kw = dict(norm=norm, branches=branches, extra_tokens=extra,
              flags=flags | (b.FLAG_KEEP_STATE if want_state else 0))
    if fused_layout:
        qkv = torch.empty((B, N, 3, H, d), dtype=x["q"].dtype, device=dev)
        for i, n in enumerate(("q", "k", "v")):
            qkv[:, :, i] = x[n].to(dev).permute(0, 2, 1, 3)
        q, k, v = (qkv[:, :, i] for i in range(3))
        out = torch.full((B, N, H * d), float("nan"), dtype=x["q"].dtype, device=dev)
        attn = b.CastlingAttn.for_workload(wl, in_strides=b.fused_qkv_strides(H, N, d),
                                           out_strides=b.token_major_strides(H, N, d), **kw)
    else:
        q, k, v = (x[n].to(dev) for n in ("q", "k", "v"))
        out = torch.full_like(q, float("nan"))
        attn = b.CastlingAttn.for_workload(wl, **kw)
    attn.forward(q, k, v, w, bias, out)
    torch.cuda.synchronize()
    st = attn.get_state() if want_state else None
    launches = attn.num_launches()
    attn.destroy()
    if fused_layout:
        out = out.view(B, N, H, d).permute(0, 2, 1, 3).contiguous()
    return inputs.to_f64(out), st, launches


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"{c[0].name}+{c[1]}")
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_class_tokens_against_definition(oracle, case, norm):
    wl, extra = case
    x = draw(wl, extra, seed=51)
    q, k, v, w, bias = oracle_inputs(x)
    for branches in (b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        print(f"case class tokens {wl.name}+{extra} norm={norm} branches={branches}", flush=True)
        want = oracle.forward_explicit(q, k, v, w, bias, wl.grid_h, wl.grid_w, norm=norm,
                                       branches=branches, extra=extra)
        lin = bool(branches & b.BRANCH_LINEAR)
        got, st, _ = run(wl, extra, x, norm, branches, want_state=lin)
        assert np.isfinite(got).all()
        assert rel_err(got, want) <= TOL[wl.dtype], (wl.name, norm, branches)
        # the class tokens alone, against their own scale
        assert rel_err(got[:, :, :extra], want[:, :, :extra]) <= TOL[wl.dtype]
        if not lin:
            assert not got[:, :, :extra].any()               # no convolution off the grid
        else:
            assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]


@pytest.mark.parametrize("case", CASES[:4], ids=lambda c: f"{c[0].name}+{c[1]}")
def test_class_tokens_strided_layout(case):
    wl, extra = case
    x = draw(wl, extra, seed=52)
    dense, _, n1 = run(wl, extra, x, b.NORM_ROWSUM, b.BRANCH_ALL)
    fused, _, n2 = run(wl, extra, x, b.NORM_ROWSUM, b.BRANCH_ALL, fused_layout=True)
    assert np.array_equal(dense, fused) and n1 == n2


def test_class_token_paths_and_validation():
    # 14 x 14 + 1 fits the one-kernel path; kept on the two-pass kernels it costs one launch more
    wl, extra = CASES[0]
    x = draw(wl, extra, seed=53)
    one, _, n_one = run(wl, extra, x, b.NORM_ROWSUM, b.BRANCH_ALL)
    assert n_one == 1
    two, _, n_two = run(wl, extra, x, b.NORM_ROWSUM, b.BRANCH_ALL, flags=b.FLAG_SEPARATE_PASSES)
    assert n_two == 4                   # reduce, combine, apply (grid), apply (class tokens)
    assert rel_err(one, two) <= 2.0 ** -7
    bad = b.make_desc(1, 1, 196, 64, 14, 14, 3, "bf16", extra_tokens=1)   # N must be 197
    assert b.validate(bad) == b.ERR_INVALID_ARG
    assert b.validate(b.make_desc(1, 1, 197, 64, 14, 14, 3, "bf16", extra_tokens=1)) == b.OK
    assert b.validate(b.make_desc(1, 1, 195, 64, 14, 14, 3, "bf16", extra_tokens=-1)) == b.ERR_INVALID_ARG
    assert b.validate(b.make_desc(1, 1, 296, 64, 14, 14, 3, "bf16", extra_tokens=100)) == b.ERR_INVALID_ARG
