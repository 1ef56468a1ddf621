"""GPU parity of downsampling attention layers (Sec. 3.1 and the last row of Table 1 of the
paper): queries pooled after their projection (q_pool = 2: one query per second row and column
of the token grid), K and V on every token, the pooled query added back (RESIDUAL_Q).  The HIP
path through the C ABI against the oracle's definition of the same layer."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import STATE_TOL, TOL, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# every I/O type and kernel width, odd grids (the coarse grid rounds up), grids narrower than
# the filter, head widths between the kernels' own, many token splits per unit in pass 1
CASES = [
    Workload("ds_bf16_d64_14x14_k3", "bf16", 2, 3, 64, 14, 14, 3),
    Workload("ds_bf16_d64_13x19_k5", "bf16", 1, 2, 64, 13, 19, 5),
    Workload("ds_f32_d32_10x17_k3", "f32", 2, 2, 32, 10, 17, 3),
    Workload("ds_f16_d64_20x36_k7", "f16", 1, 3, 64, 20, 36, 7),
    Workload("ds_bf16_d96_14x14_k3", "bf16", 1, 4, 96, 14, 14, 3),
    Workload("ds_f32_d128_6x8_k3", "f32", 1, 2, 128, 6, 8, 3),
    Workload("ds_bf16_d32_28x28_k3", "bf16", 1, 4, 32, 28, 28, 3),
    Workload("ds_bf16_d16_9x9_k9", "bf16", 1, 2, 16, 9, 9, 9),
    Workload("ds_f16_d128_5x3_k5", "f16", 2, 1, 128, 5, 3, 5),
    Workload("ds_bf16_d64_1x37_k3", "bf16", 1, 2, 64, 1, 37, 3),
    Workload("ds_bf16_d64_56x56_k3", "bf16", 1, 2, 64, 56, 56, 3),
    Workload("ds_f32_d64_33x40_k1", "f32", 1, 1, 64, 33, 40, 1),
]


def coarse(wl):
    return Workload(wl.name + "_q", wl.dtype, wl.B, wl.heads, wl.d, -(-wl.grid_h // 2),
                    -(-wl.grid_w // 2), wl.dw_kernel)


def draw(wl, seed):
    """K, V, filters on the token grid; the pooled queries drawn on the coarse grid."""
    x = inputs.make_inputs(wl, seed=seed, with_bias=True)
    x["q"] = inputs.make_inputs(coarse(wl), seed=seed + 1000)["q"]
    return x


def run(wl, x, pool=2, residual=True, norm=b.NORM_ROWSUM, branches=b.BRANCH_ALL, want_state=False):
    dev = torch.device("cuda:0")
    t = {n: (None if x[n] is None else x[n].to(dev)) for n in ("q", "k", "v", "w", "bias")}
    out = torch.full_like(t["q"], float("nan"))
    flags = (b.FLAG_RESIDUAL_Q if residual else 0) | (b.FLAG_KEEP_STATE if want_state else 0)
    attn = b.CastlingAttn(b.make_desc(wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel,
                                      wl.dtype, norm, branches, flags=flags, q_pool=pool))
    attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], out)
    torch.cuda.synchronize()
    st = attn.get_state() if want_state else None
    launches = attn.num_launches()
    attn.destroy()
    return inputs.to_f64(out), st, launches


@pytest.mark.parametrize("wl", CASES, ids=lambda w: w.name)
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_downsampling_layer_against_definition(oracle, wl, norm):
    x = draw(wl, seed=71)
    q, k, v, w, bias = oracle_inputs(x)
    for branches, residual in ((b.BRANCH_ALL, True), (b.BRANCH_ALL, False), (b.BRANCH_LINEAR, True),
                               (b.BRANCH_DWCONV, False)):
        print(f"case downsampling {wl.name} norm={norm} branches={branches} res={residual}", flush=True)
        want = oracle.forward_pooled_explicit(q, k, v, w, bias, wl.grid_h, wl.grid_w, pool=2,
                                              residual=residual, norm=norm, branches=branches)
        lin = bool(branches & b.BRANCH_LINEAR)
        got, st, _ = run(wl, x, residual=residual, norm=norm, branches=branches, want_state=lin)
        assert got.shape == want.shape and np.isfinite(got).all()
        assert rel_err(got, want) <= TOL[wl.dtype], (wl.name, norm, branches, residual)
        if lin:
            assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]


RESIDUAL_ONLY = [
    (Workload("rq_bf16_d64_14x14_k3", "bf16", 2, 3, 64, 14, 14, 3), 0),
    (Workload("rq_bf16_d64_14x14_k3_cls", "bf16", 1, 2, 64, 14, 14, 3), 1),
    (Workload("rq_f32_d32_9x21_k5", "f32", 1, 2, 32, 9, 21, 5), 0),
    (Workload("rq_f16_d32_20x24_k3", "f16", 1, 4, 32, 20, 24, 3), 2),
    (Workload("rq_bf16_d64_40x44_k9", "bf16", 1, 2, 64, 40, 44, 9), 0),
]


@pytest.mark.parametrize("case", RESIDUAL_ONLY, ids=lambda c: f"{c[0].name}+{c[1]}")
def test_residual_query_without_pooling(oracle, case):
    """One query per token plus the residual connection: the layer's output plus q, class
    tokens included."""
    wl, extra = case
    flat = Workload(wl.name, wl.dtype, wl.B, wl.heads, wl.d, 1, wl.N + extra, wl.dw_kernel)
    x = inputs.make_inputs(flat, seed=72, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    print(f"case residual query {wl.name}+{extra}", flush=True)
    want = oracle.forward_explicit(q, k, v, w, bias, wl.grid_h, wl.grid_w, extra=extra) + q
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}
    out = torch.full_like(t["q"], float("nan"))
    attn = b.CastlingAttn(b.make_desc(wl.B, wl.heads, wl.N + extra, wl.d, wl.grid_h, wl.grid_w,
                                      wl.dw_kernel, wl.dtype, flags=b.FLAG_RESIDUAL_Q,
                                      extra_tokens=extra))
    attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], out)
    torch.cuda.synchronize()
    attn.destroy()
    assert rel_err(inputs.to_f64(out), want) <= TOL[wl.dtype]


@pytest.mark.parametrize("wl", [CASES[0], CASES[2], CASES[4], CASES[10]], ids=lambda w: w.name)
def test_downsampling_layer_in_projection_adjacent_layouts(oracle, wl):
    """q as [B][Nq][heads][d] (what a pooling operator over token-major queries leaves), k and v
    as slices of one fused [B][N][2][heads][d] tensor, out as [B][Nq][heads * d]; the padding
    between rows holds NaN and must not be read."""
    x = draw(wl, seed=73)
    dev = torch.device("cuda:0")
    B, H, N, d = wl.B, wl.heads, wl.N, wl.d
    nq = coarse(wl).N
    dt = x["q"].dtype
    kv = torch.full((B, N, 2, H, d), float("nan"), dtype=dt, device=dev)
    kv[:, :, 0] = x["k"].to(dev).permute(0, 2, 1, 3)
    kv[:, :, 1] = x["v"].to(dev).permute(0, 2, 1, 3)
    pad = 8
    qt = torch.full((B, nq, H, d + pad), float("nan"), dtype=dt, device=dev)
    qt[..., :d] = x["q"].to(dev).permute(0, 2, 1, 3)
    out = torch.full((B, nq, H * d), float("nan"), dtype=dt, device=dev)
    print(f"case downsampling layouts {wl.name}", flush=True)
    attn = b.CastlingAttn(b.make_desc(
        B, H, N, d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype, flags=b.FLAG_RESIDUAL_Q, q_pool=2,
        in_strides=(N * 2 * H * d, d, 2 * H * d), q_strides=(nq * H * (d + pad), d + pad, H * (d + pad)),
        out_strides=b.token_major_strides(H, nq, d)))
    attn.forward(qt[..., :d], kv[:, :, 0], kv[:, :, 1], x["w"].to(dev), x["bias"].to(dev), out)
    torch.cuda.synchronize()
    attn.destroy()
    got = inputs.to_f64(out.view(B, nq, H, d).permute(0, 2, 1, 3).contiguous())
    dense, _, _ = run(wl, x)
    assert np.array_equal(got, dense)  # the same kernels on the same values
    q, k, v, w, bias = oracle_inputs(x)
    want = oracle.forward_pooled(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    assert rel_err(got, want) <= TOL[wl.dtype]


def test_reduce_then_apply_with_pooled_queries(oracle):
    wl = CASES[1]
    x = draw(wl, seed=74)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}
    whole, _, _ = run(wl, x)
    attn = b.CastlingAttn(b.make_desc(wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel,
                                      wl.dtype, flags=b.FLAG_RESIDUAL_Q, q_pool=2))
    out = torch.full_like(t["q"], float("nan"))
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], t["w"], t["bias"], out)
    torch.cuda.synchronize()
    # out may not overlap the pooled q; it is far smaller than k and v
    with pytest.raises(b.CastlingError) as e:
        attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], t["q"])
    assert e.value.status == b.ERR_ALIAS
    attn.destroy()
    q, k, v, w, bias = oracle_inputs(x)
    assert rel_err(inputs.to_f64(out), oracle.forward_pooled(q, k, v, w, bias, wl.grid_h, wl.grid_w)) \
        <= TOL[wl.dtype]
    assert rel_err(inputs.to_f64(out), whole) <= TOL[wl.dtype]


def test_shapes_whose_tile_of_v_exceeds_the_lds_are_refused():
    # 4 x 16 queries of stride 2 under a 9 x 9 filter read 15 x 39 tokens of V: 300 KB at
    # 128 fp32 channels, more than a compute unit holds
    d = b.make_desc(1, 1, 64 * 64, 128, 64, 64, 9, "f32", q_pool=2)
    assert b.validate(d) == b.OK
    with pytest.raises(b.CastlingError) as e:
        b.CastlingAttn(d)
    assert e.value.status == b.ERR_UNSUPPORTED
    b.CastlingAttn(b.make_desc(1, 1, 64 * 64, 128, 64, 64, 3, "f32", q_pool=2)).destroy()


# ---------------------------------------------------------------- backward of the downsampling layer
from parity_util import GRAD_TOL  # noqa: E402

BACKWARD = [CASES[0], CASES[1], CASES[2], CASES[3], CASES[4], CASES[6], CASES[8],
            Workload("ds_bf16_d64_30x34_k5", "bf16", 1, 2, 64, 30, 34, 5)]


def run_backward(wl, x, g, residual=True, norm=b.NORM_ROWSUM, branches=b.BRANCH_ALL, fused=False):
    dev = torch.device("cuda:0")
    B, H, N, d = wl.B, wl.heads, wl.N, wl.d
    nq = coarse(wl).N
    flags = b.FLAG_TRAINING | (b.FLAG_RESIDUAL_Q if residual else 0)
    kw = dict(norm=norm, branches=branches, flags=flags, q_pool=2)
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    t["g"] = g.to(dev)
    if fused:  # q, g token-major; k, v slices of one fused tensor, and so their gradients
        dt = x["q"].dtype
        kv = torch.full((B, N, 2, H, d), float("nan"), dtype=dt, device=dev)
        kv[:, :, 0], kv[:, :, 1] = (x[n].to(dev).permute(0, 2, 1, 3) for n in ("k", "v"))
        t["k"], t["v"] = kv[:, :, 0], kv[:, :, 1]
        t["q"] = x["q"].to(dev).permute(0, 2, 1, 3).contiguous()
        t["g"] = g.to(dev).permute(0, 2, 1, 3).contiguous()
        dkv = torch.full_like(kv, float("nan"))
        gk, gv = dkv[:, :, 0], dkv[:, :, 1]
        gq = torch.full_like(t["q"], float("nan"))
        kw.update(in_strides=(N * 2 * H * d, d, 2 * H * d), q_strides=b.token_major_strides(H, nq, d),
                  out_strides=b.token_major_strides(H, nq, d))
    else:
        gq = torch.full_like(t["q"], float("nan"))
        gk, gv = (torch.full_like(t["k"], float("nan")) for _ in range(2))
    gw = torch.full(t["w"].shape, float("nan"), dtype=torch.float32, device=dev)
    gb = torch.full((H, d), float("nan"), dtype=torch.float32, device=dev)
    attn = b.CastlingAttn(b.make_desc(B, H, N, d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype, **kw))
    outs = []
    for rep in range(2):  # the buffers that hold rows on the fine grid are reused as they are
        attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], gq, gk, gv, gw, gb)
        torch.cuda.synchronize()
        res = [a.permute(0, 2, 1, 3).contiguous() if fused else a for a in (gq, gk, gv)]
        outs.append([inputs.to_f64(a) for a in res] + [gw.double().cpu().numpy(), gb.double().cpu().numpy()])
    attn.destroy()
    assert all(np.array_equal(a, c) for a, c in zip(outs[0], outs[1]))
    return outs[0]


@pytest.mark.parametrize("wl", BACKWARD, ids=lambda w: w.name)
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_downsampling_backward_against_definition(oracle, wl, norm):
    x = draw(wl, seed=75)
    g = inputs.make_inputs(coarse(wl), seed=1075)["v"]
    q, k, v, w, _ = oracle_inputs(x)
    for branches, residual in ((b.BRANCH_ALL, True), (b.BRANCH_LINEAR, False), (b.BRANCH_DWCONV, False)):
        print(f"case downsampling backward {wl.name} norm={norm} branches={branches}", flush=True)
        want = oracle.backward_pooled_explicit(q, k, v, w, inputs.to_f64(g), wl.grid_h, wl.grid_w,
                                               residual=residual, norm=norm, branches=branches)
        got = run_backward(wl, x, g, residual=residual, norm=norm, branches=branches)
        for name, a, o in zip(("dq", "dk", "dv", "dw", "dbias"), got, want):
            assert np.isfinite(a).all(), (wl.name, name)
            if np.sqrt(np.mean(o * o)) < 1e-9:
                assert np.abs(a).max() < 2e-3, (wl.name, name)
                continue
            err = rel_err(a, o)
            print(f"  {name} err {err:.2e}", flush=True)
            assert err <= GRAD_TOL[wl.dtype], (wl.name, norm, branches, name, err)


@pytest.mark.parametrize("wl", [CASES[0], CASES[2], CASES[4]], ids=lambda w: w.name)
def test_downsampling_backward_in_projection_adjacent_layouts(oracle, wl):
    x = draw(wl, seed=76)
    g = inputs.make_inputs(coarse(wl), seed=1076)["v"]
    q, k, v, w, _ = oracle_inputs(x)
    print(f"case downsampling backward layouts {wl.name}", flush=True)
    want = oracle.backward_pooled_explicit(q, k, v, w, inputs.to_f64(g), wl.grid_h, wl.grid_w)
    got = run_backward(wl, x, g, fused=True)
    for name, a, o in zip(("dq", "dk", "dv", "dw", "dbias"), got, want):
        assert rel_err(a, o) <= GRAD_TOL[wl.dtype], (wl.name, name)
