"""GPU parity of the backward pass: castling_attn_backward through the C ABI against the
oracle's gradients (derivatives of the forward definition, themselves pinned to autograd and to
finite differences) on the same seeded inputs.  Each gradient tensor is held to the layer's
gradient tolerance for its I/O type (parity_util.GRAD_TOL), error = max |g - o| / max(|o|, rms(o))."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import GRAD_TOL, TOL, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# every kernel family of the forward passes the backward reuses: vector ALU (fp32, d = 16 / 128,
# padded widths), matrix cores (16-bit d = 64), pairs of 32-wide heads; ragged grids, grids
# narrower than the filter, several token splits per unit
CASES = [
    Workload("bw_f32_d32_14x14_k3", "f32", 2, 2, 32, 14, 14, 3),
    Workload("bw_bf16_d64_13x19_k5", "bf16", 2, 3, 64, 13, 19, 5),
    Workload("bw_bf16_d32_20x24_k3_pairs", "bf16", 1, 4, 32, 20, 24, 3),
    Workload("bw_f16_d64_10x17_k7", "f16", 1, 2, 64, 10, 17, 7),
    Workload("bw_f32_d128_6x8_k3", "f32", 1, 2, 128, 6, 8, 3),
    Workload("bw_bf16_d96_9x9_k3", "bf16", 1, 2, 96, 9, 9, 3),
    Workload("bw_f32_d16_5x33_k9", "f32", 1, 3, 16, 5, 33, 9),
    Workload("bw_bf16_d64_3x3_k9", "bf16", 1, 2, 64, 3, 3, 9),
    Workload("bw_bf16_d64_40x44_k5", "bf16", 1, 2, 64, 40, 44, 5),
    Workload("bw_f32_d64_33x40_k1", "f32", 1, 1, 64, 33, 40, 1),
    Workload("bw_f16_d32_7x9_k5_odd_heads", "f16", 1, 3, 32, 7, 9, 5),
]


def draw(wl, extra, seed):
    flat = Workload(wl.name, wl.dtype, wl.B, wl.heads, wl.d, 1, wl.N + extra, wl.dw_kernel)
    x = inputs.make_inputs(flat, seed=seed, with_bias=True)
    x["g"] = inputs.make_inputs(flat, seed=seed + 500)["v"]
    return x


def run(wl, x, extra=0, norm=b.NORM_ROWSUM, branches=b.BRANCH_ALL, residual=False, want_bias=True,
        layout="dense"):
    dev = torch.device("cuda:0")
    B, H, N, d = wl.B, wl.heads, wl.N + extra, wl.d
    dt = x["q"].dtype
    flags = b.FLAG_TRAINING | (b.FLAG_RESIDUAL_Q if residual else 0)
    kw = dict(norm=norm, branches=branches, flags=flags, extra_tokens=extra)
    if layout == "dense":
        t = {n: x[n].to(dev) for n in ("q", "k", "v", "g")}
        grads = [torch.full_like(t["q"], float("nan")) for _ in range(3)]
        views = grads
    else:  # q, k, v and their gradients as slices of fused [B][N][3][heads][d] tensors
        qkv = torch.full((B, N, 3, H, d), float("nan"), dtype=dt, device=dev)
        for i, n in enumerate(("q", "k", "v")):
            qkv[:, :, i] = x[n].to(dev).permute(0, 2, 1, 3)
        t = {n: qkv[:, :, i] for i, n in enumerate(("q", "k", "v"))}
        t["g"] = x["g"].to(dev).permute(0, 2, 1, 3).contiguous()  # [B][N][heads][d]
        dqkv = torch.full_like(qkv, float("nan"))
        views = [dqkv[:, :, i] for i in range(3)]
        kw.update(in_strides=b.fused_qkv_strides(H, N, d), out_strides=b.token_major_strides(H, N, d))
    w = x["w"].to(dev)
    gw = torch.full(w.shape, float("nan"), dtype=torch.float32, device=dev)
    gb = torch.full((H, d), float("nan"), dtype=torch.float32, device=dev) if want_bias else None
    attn = b.CastlingAttn(b.make_desc(B, H, N, d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype, **kw))
    attn.backward(t["q"], t["k"], t["v"], w, t["g"], views[0], views[1], views[2], gw, gb)
    torch.cuda.synchronize()
    attn.destroy()
    if layout == "dense":
        out = [inputs.to_f64(a) for a in views]
    else:
        out = [inputs.to_f64(a.permute(0, 2, 1, 3).contiguous()) for a in views]
    return out + [gw.double().cpu().numpy(), None if gb is None else gb.double().cpu().numpy()]


def check(got, want, tol, tag):
    for name, a, o in zip(("dq", "dk", "dv", "dw", "dbias"), got, want):
        if o is None:
            assert a is None
            continue
        assert np.isfinite(a).all(), (tag, name)
        if np.sqrt(np.mean(o * o)) < 1e-9:
            # a gradient that vanishes identically (one token: the output does not depend on q, k):
            # there is no scale to be relative to: terms of order one cancel, to fp32 rounding
            # with fp32 I/O and to that of the 16-bit operands otherwise
            assert np.abs(a).max() < (1e-5 if tol <= 1e-4 else 2e-3), (tag, name)
            continue
        err = rel_err(a, o)
        print(f"  {name} err {err:.2e}", flush=True)
        assert err <= tol, (tag, name, err)


@pytest.mark.parametrize("wl", CASES, ids=lambda w: w.name)
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_gradients_against_the_definition(oracle, wl, norm):
    x = draw(wl, 0, seed=91)
    q, k, v, w, _ = oracle_inputs(x)
    g = inputs.to_f64(x["g"])
    for branches in (b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        print(f"case backward {wl.name} norm={norm} branches={branches}", flush=True)
        want = oracle.backward_explicit(q, k, v, w, g, wl.grid_h, wl.grid_w, norm=norm,
                                        branches=branches)
        got = run(wl, x, norm=norm, branches=branches)
        check(got, want, GRAD_TOL[wl.dtype], (wl.name, norm, branches))


EXTRAS = [(CASES[0], 1, False), (CASES[1], 2, True), (CASES[2], 1, True), (CASES[5], 1, False),
          (CASES[3], 0, True)]


@pytest.mark.parametrize("case", EXTRAS, ids=lambda c: f"{c[0].name}+{c[1]}{'+res' if c[2] else ''}")
def test_gradients_with_class_tokens_and_residual_query(oracle, case):
    wl, extra, residual = case
    x = draw(wl, extra, seed=92)
    q, k, v, w, _ = oracle_inputs(x)
    g = inputs.to_f64(x["g"])
    print(f"case backward {wl.name} extra={extra} residual={residual}", flush=True)
    want = oracle.backward_explicit(q, k, v, w, g, wl.grid_h, wl.grid_w, extra=extra,
                                    residual=residual, with_bias=False)
    got = run(wl, x, extra=extra, residual=residual, want_bias=False)
    check(got, want, GRAD_TOL[wl.dtype], (wl.name, extra, residual))


@pytest.mark.parametrize("wl", [CASES[0], CASES[1], CASES[2], CASES[8]], ids=lambda w: w.name)
def test_gradients_in_projection_adjacent_layouts(oracle, wl):
    """The gradients of q, k, v land in the slices of one fused tensor, ready for the backward
    of the QKV projection; grad_out comes token-major from the output projection's backward."""
    x = draw(wl, 0, seed=93)
    q, k, v, w, _ = oracle_inputs(x)
    print(f"case backward layouts {wl.name}", flush=True)
    want = oracle.backward(q, k, v, w, inputs.to_f64(x["g"]), wl.grid_h, wl.grid_w)
    got = run(wl, x, layout="fused")
    check(got, want, GRAD_TOL[wl.dtype], wl.name)


def test_rows_under_the_norm_floor_and_repeat_calls(oracle):
    wl = CASES[0]
    x = draw(wl, 0, seed=94)
    x["q"][:, :, 5] = 0
    x["k"][:, :, 7] = 0
    x["q"][:, :, 9] *= 1e-3
    q, k, v, w, _ = oracle_inputs(x)
    g = inputs.to_f64(x["g"])
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "g", "w")}
    attn = b.CastlingAttn(b.make_desc(wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel,
                                      wl.dtype, eps=1e-2, flags=b.FLAG_TRAINING))
    want = oracle.backward_explicit(q, k, v, w, g, wl.grid_h, wl.grid_w, eps=1e-2)
    outs = []
    for rep in range(2):  # a forward in between leaves the backward's result unchanged
        gq, gk, gv = (torch.full_like(t["q"], float("nan")) for _ in range(3))
        gw = torch.empty(t["w"].shape, dtype=torch.float32, device=dev)
        gb = torch.empty((wl.heads, wl.d), dtype=torch.float32, device=dev)
        attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], gq, gk, gv, gw, gb)
        fwd = torch.empty_like(t["q"])
        attn.forward(t["q"], t["k"], t["v"], t["w"], None, fwd)
        torch.cuda.synchronize()
        outs.append([inputs.to_f64(a) for a in (gq, gk, gv)] + [gw.double().cpu().numpy(),
                                                                gb.double().cpu().numpy()])
        check(outs[-1], want, GRAD_TOL[wl.dtype], ("floor", rep))
    assert all(np.array_equal(a, c) for a, c in zip(outs[0], outs[1]))
    assert rel_err(inputs.to_f64(fwd), oracle.forward(q, k, v, w, None, wl.grid_h, wl.grid_w, eps=1e-2)) \
        <= TOL[wl.dtype]
    # after a backward the handle holds no state of (k, v)
    with pytest.raises(b.CastlingError):
        attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], gq, gk, gv, gw, gb)
        attn.get_state()
    attn.destroy()


def test_backward_needs_a_training_handle_and_distinct_buffers():
    wl = CASES[0]
    x = draw(wl, 0, seed=95)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "g", "w")}
    gq, gk, gv = (torch.empty_like(t["q"]) for _ in range(3))
    gw = torch.empty(t["w"].shape, dtype=torch.float32, device=dev)
    plain = b.CastlingAttn.for_workload(wl)
    with pytest.raises(b.CastlingError) as e:
        plain.backward(t["q"], t["k"], t["v"], t["w"], t["g"], gq, gk, gv, gw)
    assert e.value.status == b.ERR_INVALID_ARG
    bigger = plain.workspace_bytes()
    plain.destroy()
    attn = b.CastlingAttn.for_workload(wl, flags=b.FLAG_TRAINING)
    assert attn.workspace_bytes() > bigger
    with pytest.raises(b.CastlingError) as e:
        attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], t["q"], gk, gv, gw)
    assert e.value.status == b.ERR_ALIAS
    with pytest.raises(b.CastlingError) as e:
        attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], gq, gq, gv, gw)
    assert e.value.status == b.ERR_ALIAS
    with pytest.raises(b.CastlingError) as e:
        attn.backward(t["q"], t["k"], t["v"], None, t["g"], gq, gk, gv, gw)
    assert e.value.status == b.ERR_INVALID_ARG
    # the fp32 filter and bias gradients are outputs like the others
    gb = torch.empty(t["w"].shape[:2], dtype=torch.float32, device=dev)
    as_f32 = t["q"].view(torch.float32).reshape(-1)
    bad = [dict(gw=as_f32[:gw.numel()]),                       # grad_w inside q
           dict(gw=gq.view(torch.float32).reshape(-1)[:gw.numel()]),  # grad_w inside grad_q
           dict(gb=gw.reshape(-1)[:gb.numel()]),               # grad_bias inside grad_w
           dict(gw=t["w"].view(torch.float32).reshape(-1)) if t["w"].element_size() == 4 else
           dict(gb=t["g"].view(torch.float32).reshape(-1)[:gb.numel()])]   # inside grad_out
    for kw in bad:
        with pytest.raises(b.CastlingError) as e:
            attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], gq, gk, gv, kw.get("gw", gw),
                          kw.get("gb", gb))
        assert e.value.status == b.ERR_ALIAS, list(kw)
    attn.destroy()


@pytest.mark.parametrize("name", ["cfg5_bf16_b2_h12_d64_n16384_k9", "x_f16_b2_h12_d64_n16384_k9",
                                  "cfg1_f32_b1_h4_d32_n196_k3", "cfg2_bf16_b64_h8_d64_n196_k3",
                                  "cfg3_bf16_b32_h6_d64_n784_k3_outliers",
                                  "cfg4_bf16_b8_h8_d64_n4096_k5"])
def test_gradients_at_benchmark_size(oracle, name):
    """The benchmark workloads (and the fp16 twin of the largest: a = g / den is of the order
    1e-4 there, stored scaled) in the configuration bench.py --backward times.  Every element
    against the oracle's reassociated backward, and sampled rows of dq, dk, dv against the
    gradient of the definition itself (explicit N x N similarities, nothing of the reassociated
    derivation that oracle and kernels share)."""
    wl = inputs.workload(name)
    x = draw(wl, 0, seed=96)
    q, k, v, w, _ = oracle_inputs(x)
    g = inputs.to_f64(x["g"])
    print(f"case backward full size {wl.name}", flush=True)
    want = oracle.backward(q, k, v, w, g, wl.grid_h, wl.grid_w)
    # first and last unit; corners and interior of the grid, first and last token
    N, W = wl.N, wl.grid_w
    toks = np.array([0, 1, W - 1, W, N // 2 + 3, N - W, N - 1])
    units = np.repeat([0, wl.units - 1], len(toks))
    tokens = np.tile(toks, 2)
    rows = oracle.backward_explicit_rows(q, k, v, w, g, wl.grid_h, wl.grid_w, units, tokens)
    for name_, full, r in zip(("dq", "dk", "dv"), want, rows):
        # the oracle's two forms agree at full size far below any kernel tolerance
        np.testing.assert_allclose(full.reshape(wl.units, N, wl.d)[units, tokens], r, rtol=1e-7,
                                   atol=1e-9 * np.abs(full).max(), err_msg=name_)
    got = run(wl, x)
    check(got, want, GRAD_TOL[wl.dtype], wl.name)
    for name_, a, full, r in zip(("dq", "dk", "dv"), got, want, rows):
        rms = np.sqrt(np.mean(full * full))
        err = np.max(np.abs(a.reshape(wl.units, N, wl.d)[units, tokens] - r) / np.maximum(np.abs(r), rms))
        assert err <= GRAD_TOL[wl.dtype], (wl.name, name_, err)


EDGES = [
    (Workload("bw_f32_d8_1x1_k1", "f32", 1, 1, 8, 1, 1, 1), 0),
    (Workload("bw_bf16_d64_1x1_k3", "bf16", 2, 2, 64, 1, 1, 3), 0),
    (Workload("bw_bf16_d8_6x6_k3", "bf16", 1, 3, 8, 6, 6, 3), 0),
    (Workload("bw_f16_d24_5x7_k5", "f16", 2, 1, 24, 5, 7, 5), 0),
    (Workload("bw_bf16_d64_2x2_k9_cls64", "bf16", 1, 2, 64, 2, 2, 9), 64),
    (Workload("bw_bf16_d32_1x70_k7_pairs", "bf16", 1, 2, 32, 1, 70, 7), 0),
    (Workload("bw_f32_d64_70x1_k3", "f32", 1, 1, 64, 70, 1, 3), 0),
    (Workload("bw_bf16_d64_8x8_k3_many_units", "bf16", 40, 60, 64, 8, 8, 3), 0),
]


@pytest.mark.parametrize("case", EDGES, ids=lambda c: c[0].name)
def test_gradients_at_the_edges(oracle, case):
    """One token, the narrowest heads, padded widths, the maximum number of class tokens, grids
    of one row or column, more units than the filter gradient has chunks for."""
    wl, extra = case
    x = draw(wl, extra, seed=97)
    q, k, v, w, _ = oracle_inputs(x)
    print(f"case backward edge {wl.name}", flush=True)
    want = oracle.backward(q, k, v, w, inputs.to_f64(x["g"]), wl.grid_h, wl.grid_w, extra=extra)
    got = run(wl, x, extra=extra)
    check(got, want, GRAD_TOL[wl.dtype], wl.name)


@pytest.mark.parametrize("wl", [CASES[0], CASES[1], CASES[2]], ids=lambda w: w.name)
def test_backward_in_a_captured_graph(oracle, wl):
    """backward() only enqueues kernels (no allocation, synchronisation or memset), so a
    training step can capture it in a HIP graph: every replay, with eager work and
    synchronisations in between and new inputs written into the captured buffers, reproduces
    the eager gradients bit for bit."""
    dev = torch.device("cuda:0")
    xs = [draw(wl, 0, seed=98 + i) for i in range(3)]
    names = ("q", "k", "v", "w", "g")
    bufs = {n: torch.empty_like(xs[0][n], device=dev) for n in names}

    def grads():
        return [torch.full_like(bufs["q"], float("nan")) for _ in range(3)] + \
               [torch.full(bufs["w"].shape, float("nan"), dtype=torch.float32, device=dev),
                torch.full((wl.heads, wl.d), float("nan"), dtype=torch.float32, device=dev)]

    captured, eager = grads(), grads()
    attn = b.CastlingAttn.for_workload(wl, flags=b.FLAG_TRAINING)
    side = torch.cuda.Stream()
    for n in names:
        bufs[n].copy_(xs[0][n])
    torch.cuda.synchronize()
    args = [bufs[n] for n in names]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        attn.backward(*args, *captured, stream=side)  # warm-up
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            attn.backward(*args, *captured, stream=torch.cuda.current_stream())
    for i, x in enumerate(xs):
        print(f"case backward graph replay {wl.name} #{i}", flush=True)
        for n in names:
            bufs[n].copy_(x[n])
        torch.cuda.synchronize()
        for t in captured:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        attn.backward(*args, *eager)
        torch.cuda.synchronize()
        for a, c in zip(captured, eager):
            assert torch.equal(a.view(torch.int32 if a.element_size() == 4 else torch.int16),
                               c.view(torch.int32 if c.element_size() == 4 else torch.int16))
        q, k, v, w, _ = oracle_inputs(x)
        want = oracle.backward(q, k, v, w, inputs.to_f64(x["g"]), wl.grid_h, wl.grid_w)
        got = [inputs.to_f64(t) if t.dtype != torch.float32 or wl.dtype == "f32" else t.double().cpu().numpy()
               for t in captured]
        check(got, want, GRAD_TOL[wl.dtype], (wl.name, "graph", i))
    del graph
    attn.destroy()
