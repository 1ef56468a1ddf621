"""GPU parity: the HIP layer (through the C ABI) against the CPU oracle on the
same seeded inputs.  Tolerances: max relative error 1e-4 (fp32 I/O) and 1e-2
(bf16 I/O, fp32 accumulation), error = max |g-o| / max(|o|, rms(o)), checked for
the whole layer and for each branch alone."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import STATE_TOL, TOL, gpu_forward, gpu_forward_fused, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# small shapes the oracle's explicit N x N form finishes quickly; they span several
# 4x16 tiles, ragged right/bottom edges, grids narrower than the filter, both
# dtypes, both head widths and every filter size
SMALL = [
    Workload("s_f32_d32_14x14_k3", "f32", 1, 4, 32, 14, 14, 3),
    Workload("s_f32_d64_10x17_k9", "f32", 2, 2, 64, 10, 17, 9),
    Workload("s_f32_d32_5x33_k5", "f32", 1, 3, 32, 5, 33, 5),
    Workload("s_bf16_d64_13x19_k5", "bf16", 2, 3, 64, 13, 19, 5),
    Workload("s_bf16_d32_7x9_k7", "bf16", 3, 2, 32, 7, 9, 7),
    Workload("s_bf16_d64_3x3_k9", "bf16", 1, 2, 64, 3, 3, 9),
    Workload("s_bf16_d64_1x40_k3", "bf16", 1, 1, 64, 1, 40, 3),
    Workload("s_f32_d32_37x1_k3", "f32", 1, 2, 32, 37, 1, 3),
    Workload("s_bf16_d64_1x1_k1", "bf16", 2, 2, 64, 1, 1, 1),
    Workload("s_bf16_d64_24x24_k3_outl", "bf16", 2, 2, 64, 24, 24, 3, 0.05, 8.0),
    Workload("s_bf16_d64_20x36_k7", "bf16", 1, 7, 64, 20, 36, 7),
    Workload("s_bf16_d64_33x17_k9", "bf16", 3, 1, 64, 33, 17, 9),
    Workload("s_bf16_d32_18x18_k9", "bf16", 1, 2, 32, 18, 18, 9),
    Workload("s_f32_d64_6x6_k7", "f32", 1, 2, 64, 6, 6, 7),
    # bf16, d = 64, N <= 256, k <= 5: forward() takes the one-kernel path; full and ragged
    # chunks of 64 tokens, every filter size, a wave with no tokens at all
    Workload("s_bf16_d64_16x16_k5", "bf16", 2, 3, 64, 16, 16, 5),
    Workload("s_bf16_d64_14x14_k3", "bf16", 3, 3, 64, 14, 14, 3),
    Workload("s_bf16_d64_8x9_k1", "bf16", 1, 2, 64, 8, 9, 1),
    Workload("s_bf16_d64_5x13_k5", "bf16", 1, 5, 64, 5, 13, 5),
    Workload("s_bf16_d64_2x50_k3", "bf16", 2, 1, 64, 2, 50, 3),
    Workload("s_bf16_d64_7x7_k5", "bf16", 2, 2, 64, 7, 7, 5),
    Workload("s_bf16_d64_4x64_k3", "bf16", 1, 2, 64, 4, 64, 3),
    Workload("s_bf16_d64_8x30_k5", "bf16", 1, 3, 64, 8, 30, 5),
    Workload("s_f16_d64_16x16_k3", "f16", 2, 2, 64, 16, 16, 3),
    Workload("s_f16_d64_10x10_k5", "f16", 1, 3, 64, 10, 10, 5),
]
ONE_KERNEL = [SMALL[3], SMALL[6], SMALL[8]] + SMALL[14:]

# 16-bit heads of 32 channels: pass 2 runs two neighbouring heads as one 64-channel unit on the
# matrix cores (even head counts); dense and fused layouts, several strips, ragged edges
HEAD_PAIRS = [
    Workload("hp_bf16_b2_h4_d32_20x24_k3", "bf16", 2, 4, 32, 20, 24, 3),
    Workload("hp_f16_b1_h6_d32_33x17_k9", "f16", 1, 6, 32, 33, 17, 9),
    Workload("hp_bf16_b3_h2_d32_14x14_k5", "bf16", 3, 2, 32, 14, 14, 5),
    Workload("hp_bf16_b1_h8_d32_9x40_k7_outl", "bf16", 1, 8, 32, 9, 40, 7, 0.05, 8.0),
    Workload("hp_bf16_b32_h8_d32_7x7_k3", "bf16", 32, 8, 32, 7, 7, 3),
]

# head widths 16 and 128 and fp16 I/O (vector-ALU kernels)
WIDE = [
    Workload("w_f32_d16_14x14_k3", "f32", 2, 3, 16, 14, 14, 3),
    Workload("w_bf16_d16_9x21_k5", "bf16", 1, 4, 16, 9, 21, 5),
    Workload("w_f16_d16_7x7_k7", "f16", 2, 2, 16, 7, 7, 7),
    Workload("w_f32_d128_10x12_k3", "f32", 1, 2, 128, 10, 12, 3),
    Workload("w_bf16_d128_14x14_k5", "bf16", 2, 2, 128, 14, 14, 5),
    Workload("w_f16_d128_6x20_k3", "f16", 1, 3, 128, 6, 20, 3),
    Workload("w_f16_d64_14x14_k3", "f16", 2, 4, 64, 14, 14, 3),
    Workload("w_f16_d32_13x19_k9", "f16", 1, 3, 32, 13, 19, 9),
    Workload("w_f16_d64_33x40_k5", "f16", 1, 2, 64, 33, 40, 5),
    Workload("w_f16_d64_24x24_k9_outl", "f16", 2, 2, 64, 24, 24, 9, 0.05, 8.0),
    Workload("w_f16_d64_20x36_k7", "f16", 1, 3, 64, 20, 36, 7),
    Workload("w_f16_d64_1x40_k1", "f16", 1, 2, 64, 1, 40, 1),
]

# head widths between the kernels' own (any multiple of 8 up to 128): the vector-ALU kernels run
# them at the next width of theirs with zero features in the gap; 96 is the width of the last
# stage of a pooling-attention backbone; one shape with several token splits per unit
ANY_WIDTH = [
    Workload("aw_bf16_d96_14x14_k3", "bf16", 2, 3, 96, 14, 14, 3),
    Workload("aw_f32_d96_9x21_k5", "f32", 1, 2, 96, 9, 21, 5),
    Workload("aw_f16_d96_7x7_k7", "f16", 2, 2, 96, 7, 7, 7),
    Workload("aw_bf16_d48_13x19_k9", "bf16", 1, 3, 48, 13, 19, 9),
    Workload("aw_f32_d24_14x14_k3", "f32", 2, 2, 24, 14, 14, 3),
    Workload("aw_f16_d40_10x12_k5", "f16", 1, 4, 40, 10, 12, 5),
    Workload("aw_bf16_d8_16x16_k3", "bf16", 1, 5, 8, 16, 16, 3),
    Workload("aw_f32_d8_6x20_k1", "f32", 1, 2, 8, 6, 20, 1),
    Workload("aw_bf16_d120_6x20_k3", "bf16", 1, 2, 120, 6, 20, 3),
    Workload("aw_f32_d72_5x33_k7", "f32", 1, 1, 72, 5, 33, 7),
    Workload("aw_bf16_d96_40x44_k5", "bf16", 1, 2, 96, 40, 44, 5),
    Workload("aw_f32_d56_36x40_k3", "f32", 1, 1, 56, 36, 40, 3),
]


@pytest.mark.parametrize("wl", WIDE + ANY_WIDTH, ids=lambda w: w.name)
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_wide_shapes_and_fp16(oracle, wl, norm):
    x = inputs.make_inputs(wl, seed=31, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    for branches in (b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        print(f"case {wl.name} norm={norm} branches={branches}", flush=True)
        want = oracle.forward_explicit(q, k, v, w, bias, wl.grid_h, wl.grid_w, norm=norm,
                                       branches=branches)
        if branches & b.BRANCH_LINEAR:
            got, st = gpu_forward(wl, x, norm=norm, branches=branches, want_state=True)
            assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]
        else:  # the convolution alone reduces nothing: there is no state to fetch
            got = gpu_forward(wl, x, norm=norm, branches=branches)
        assert np.isfinite(got).all()
        assert rel_err(got, want) <= TOL[wl.dtype], (wl.name, norm, branches)
    # strided views work for every kernel family
    assert np.array_equal(gpu_forward_fused(wl, x, norm=norm), gpu_forward(wl, x, norm=norm))


@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_small_against_definition(oracle, wl, norm):
    x = inputs.make_inputs(wl, seed=11, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    for branches in (b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        print(f"case {wl.name} norm={norm} branches={branches}", flush=True)
        want = oracle.forward_explicit(q, k, v, w, bias, wl.grid_h, wl.grid_w, norm=norm,
                                       branches=branches)
        got = gpu_forward(wl, x, norm=norm, branches=branches)
        assert np.isfinite(got).all()
        assert rel_err(got, want) <= TOL[wl.dtype], (wl.name, norm, branches)


# projection-adjacent layouts: q, k, v as slices of a fused [B][N][3][heads][d] tensor, out
# as [B][N][heads * d]; every kernel family (fp32 / bf16 vector-ALU, matrix-core) is covered
# shapes in which the persistent blocks of pass 2 get uneven step ranges that start and end in
# the middle of a strip column, with 3 and 5 strips per unit, and grids with more strips per
# unit than the chip has compute units
SCHEDULES = [
    Workload("p_bf16_d64_40x36_k3_u9", "bf16", 3, 3, 64, 40, 36, 3),
    Workload("p_f16_d64_29x72_k5_u8", "f16", 2, 4, 64, 29, 72, 5),
    Workload("p_bf16_d64_1x4200_k3", "bf16", 1, 1, 64, 1, 4200, 3),
    Workload("p_bf16_d64_2x4400_k9", "bf16", 1, 2, 64, 2, 4400, 9),
]


@pytest.mark.parametrize("wl", SCHEDULES, ids=lambda w: w.name)
def test_block_schedules_of_pass_two(oracle, wl):
    x = inputs.make_inputs(wl, seed=41, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    for branches in (b.BRANCH_ALL, b.BRANCH_DWCONV):
        print(f"case {wl.name} branches={branches}", flush=True)
        want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w, branches=branches)
        got = gpu_forward(wl, x, branches=branches)
        assert rel_err(got, want) <= TOL[wl.dtype], (wl.name, branches)


STRIDED = [SMALL[0], SMALL[1], SMALL[3], SMALL[4], SMALL[9], SMALL[10], SMALL[11], SMALL[15],
           Workload("s_bf16_d64_40x40_k5_b3", "bf16", 3, 5, 64, 40, 40, 5)]


@pytest.mark.parametrize("wl", STRIDED, ids=lambda w: w.name)
def test_fused_qkv_layout(oracle, wl):
    x = inputs.make_inputs(wl, seed=21, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    print(f"case fused layout {wl.name}", flush=True)
    want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    got, st = gpu_forward_fused(wl, x, want_state=True)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL[wl.dtype]
    dense, st_dense = gpu_forward(wl, x, want_state=True)
    if wl.d == 32 and wl.dtype != "f32" and wl.heads % 2 == 0:
        # pairs of narrow heads: pass 1 reduces whole pairs where their rows are adjacent (this
        # layout) and single heads otherwise, so the sums are taken in another order
        assert rel_err(st, st_dense) <= 1e-5
        assert rel_err(got, dense) <= TOL[wl.dtype]
        return
    # the same kernels in the same order: bitwise equal to the contiguous layout
    assert np.array_equal(got, dense)
    assert np.array_equal(st, st_dense)
    for branches in (b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        assert np.array_equal(gpu_forward_fused(wl, x, branches=branches),
                              gpu_forward(wl, x, branches=branches))


def test_padded_token_rows(oracle):
    # token stride larger than the packed row; the padding holds NaN and must never be read
    for wl in (SMALL[3], SMALL[0]):
        x = inputs.make_inputs(wl, seed=22)
        print(f"case padded rows {wl.name}", flush=True)
        got = gpu_forward_fused(wl, x, pad=8)
        assert np.array_equal(got, gpu_forward(wl, x))


@pytest.mark.parametrize("wl", SMALL[:6] + SMALL[10:12] + SMALL[14:16], ids=lambda w: w.name)
def test_state_against_oracle(oracle, wl):
    x = inputs.make_inputs(wl, seed=12)
    _, k, v, _, _ = oracle_inputs(x)
    print(f"case state {wl.name}", flush=True)
    _, st = gpu_forward(wl, x, want_state=True)
    want = oracle.state(k, v)
    d = wl.d
    # compare each part of the state against its own rms
    for name, sl in (("KtV", (slice(0, d), slice(0, d))), ("ksum", (slice(0, d), d)),
                     ("vsum", (d, slice(0, d))), ("count", (d, d))):
        g, o = st[(..., *sl)], want[(..., *sl)]
        assert rel_err(g, o) <= STATE_TOL[wl.dtype], (wl.name, name)


FULL_SIZE = list(inputs.WORKLOADS) + [inputs.workload("x_f16_b2_h12_d64_n16384_k9"),
                                      inputs.workload("x_f16_b64_h8_d64_n196_k3")]


@pytest.mark.parametrize("idx", range(len(FULL_SIZE)), ids=lambda i: FULL_SIZE[i].name)
def test_benchmark_workload_full_size(oracle, idx):
    """The five benchmark workloads (and the fp16 twins of the largest and of the one-kernel
    case) at full size: every element against the oracle's reassociated form (itself pinned
    to the definition), sampled rows against the definition, per branch, plus the exported
    state."""
    wl = FULL_SIZE[idx]
    print(f"case full {wl.name}", flush=True)
    x = inputs.make_inputs(wl)
    q, k, v, w, bias = oracle_inputs(x)
    tol = TOL[wl.dtype]
    rs = np.random.default_rng(100 + idx)
    units = rs.integers(0, wl.units, size=48)
    tokens = rs.integers(0, wl.N, size=48)
    # corners and edges of the grid are always among the samples
    tokens[:4] = [0, wl.grid_w - 1, wl.N - wl.grid_w, wl.N - 1]
    for branches in (b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        got = gpu_forward(wl, x, branches=branches)
        want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w, branches=branches)
        assert rel_err(got, want) <= tol, (wl.name, branches)
        rows = oracle.forward_explicit_rows(q, k, v, w, bias, wl.grid_h, wl.grid_w, units, tokens,
                                            branches=branches)
        rms = float(np.sqrt(np.mean(want * want)))
        g = got.reshape(wl.units, wl.N, wl.d)[units, tokens]
        err = np.max(np.abs(g - rows) / np.maximum(np.abs(rows), rms))
        assert err <= tol, (wl.name, branches, "sampled rows vs definition")
        print(f"  branches={branches} rel_err={rel_err(got, want):.3e} sampled={err:.3e}", flush=True)
    _, st = gpu_forward(wl, x, want_state=True)
    want_st = oracle.state(k, v)
    d = wl.d
    stol = STATE_TOL[wl.dtype]
    assert rel_err(st[..., :d, :d], want_st[..., :d, :d]) <= stol
    assert rel_err(st[..., :d, d], want_st[..., :d, d]) <= stol
    assert rel_err(st[..., d, :d], want_st[..., d, :d]) <= stol


def test_outlier_scaling_leaves_weights_unchanged(oracle):
    """Scaling q and k rows by positive factors must not change the linear branch."""
    wl = Workload("inv_bf16", "bf16", 1, 2, 64, 12, 20, 3)
    x = inputs.make_inputs(wl, seed=5)
    base = gpu_forward(wl, x, branches=b.BRANCH_LINEAR)
    x2 = dict(x)
    scale = torch.where(torch.rand(1, 1, wl.N, 1, generator=torch.Generator().manual_seed(1)) < 0.2,
                        torch.tensor(8.0), torch.tensor(1.0))          # powers of two: exact in bf16
    x2["q"] = (x["q"].float() * scale).to(torch.bfloat16)
    x2["k"] = (x["k"].float() * scale).to(torch.bfloat16)
    got = gpu_forward(wl, x2, branches=b.BRANCH_LINEAR)
    assert rel_err(got, base) <= 1e-3


def test_zero_rows_and_constant_v(oracle):
    wl = Workload("edge_f32", "f32", 1, 2, 32, 6, 10, 3)
    x = inputs.make_inputs(wl, seed=6)
    x["q"][0, 0, 7] = 0.0          # zero query: uniform weights -> mean of V
    x["k"][0, 1, 3] = 0.0          # zero key: weight exactly 1/2
    q, k, v, w, bias = oracle_inputs(x)
    got = gpu_forward(wl, x, branches=b.BRANCH_LINEAR)
    want = oracle.forward_explicit(q, k, v, w, None, wl.grid_h, wl.grid_w, branches=1)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= 1e-4
    np.testing.assert_allclose(got[0, 0, 7], v[0, 0].mean(axis=0), rtol=1e-4, atol=1e-6)
    x["v"][...] = 2.5
    got = gpu_forward(wl, x, branches=b.BRANCH_LINEAR)
    np.testing.assert_allclose(got, 2.5, rtol=1e-5)


@pytest.mark.parametrize("idx", [0, 2, 4])
def test_bitwise_deterministic(idx):
    wl = inputs.WORKLOADS[idx]
    print(f"case determinism {wl.name}", flush=True)
    x = inputs.make_inputs(wl)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    attn = b.CastlingAttn.for_workload(wl)
    outs = []
    for _ in range(3):
        out = torch.empty_like(t["q"])
        attn.forward(t["q"], t["k"], t["v"], t["w"], None, out)
        torch.cuda.synchronize()
        outs.append(out.view(torch.int16 if wl.dtype == "bf16" else torch.int32).cpu())
    attn.destroy()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_zero_rows_bf16(oracle):
    """bf16 path: a zero query gives uniform weights, a zero key has weight exactly 1/2."""
    wl = Workload("edge_bf16", "bf16", 2, 2, 64, 9, 18, 5)
    x = inputs.make_inputs(wl, seed=16)
    x["q"][1, 0, 40] = 0.0
    x["k"][0, 1, 3] = 0.0
    q, k, v, w, bias = oracle_inputs(x)
    got = gpu_forward(wl, x, branches=b.BRANCH_LINEAR)
    want = oracle.forward_explicit(q, k, v, w, None, wl.grid_h, wl.grid_w, branches=1)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= 1e-2
    np.testing.assert_allclose(got[1, 0, 40], v[1, 0].mean(axis=0), rtol=2e-2, atol=2e-3)


def test_forced_generic_bf16_matches_oracle(oracle):
    """The vector-ALU kernels stay reachable for bf16 (they are the fallback path)."""
    wl = SMALL[3]
    x = inputs.make_inputs(wl, seed=17, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    got = gpu_forward(wl, x, flags=b.FLAG_VECTOR_ALU)
    want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    assert rel_err(got, want) <= TOL[wl.dtype]


@pytest.mark.parametrize("wl", ONE_KERNEL + [HEAD_PAIRS[2], HEAD_PAIRS[4]], ids=lambda w: w.name)
def test_two_pass_path_at_small_n(oracle, wl):
    """Shapes that forward() would run in one kernel, kept on the reduce + apply kernels."""
    x = inputs.make_inputs(wl, seed=23, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    print(f"case two-pass {wl.name}", flush=True)
    want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    assert rel_err(gpu_forward(wl, x, flags=b.FLAG_SEPARATE_PASSES), want) <= TOL[wl.dtype]


@pytest.mark.parametrize("wl", ONE_KERNEL, ids=lambda w: w.name)
def test_one_kernel_forward_agrees_with_reduce_apply(wl):
    """forward() in one kernel against reduce() + apply() on the same handle: the same
    arithmetic up to summation order, so they agree far inside the oracle tolerance."""
    x = inputs.make_inputs(wl, seed=24, with_bias=True)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}
    plain = b.CastlingAttn.for_workload(wl)
    with pytest.raises(b.CastlingError):      # nothing has run yet
        plain.get_state()
    plain.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], torch.empty_like(t["q"]))
    with pytest.raises(b.CastlingError):      # the state stayed on chip
        plain.get_state()
    plain.destroy()
    attn = b.CastlingAttn.for_workload(wl, flags=b.FLAG_KEEP_STATE)
    o1, o2 = torch.empty_like(t["q"]), torch.empty_like(t["q"])
    print(f"case one-kernel vs two-pass {wl.name}", flush=True)
    attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], o1)
    s1 = attn.get_state()
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], t["w"], t["bias"], o2)
    s2 = attn.get_state()
    attn.destroy()
    assert rel_err(inputs.to_f64(o1), inputs.to_f64(o2)) <= 2.0 ** -7  # two bf16 roundings apart
    # same products, different summation order inside and across the matrix instructions
    assert rel_err(s1, s2) <= 1e-4


def test_reduce_then_apply_equals_forward():
    """forward() as separate launches is reduce() followed by apply(): bitwise the same."""
    wl = Workload("split_bf16", "bf16", 2, 2, 64, 19, 21, 5)
    x = inputs.make_inputs(wl, seed=8)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    attn = b.CastlingAttn.for_workload(wl, flags=b.FLAG_SEPARATE_PASSES)
    o1, o2 = torch.empty_like(t["q"]), torch.empty_like(t["q"])
    attn.forward(t["q"], t["k"], t["v"], t["w"], None, o1)
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], t["w"], None, o2)
    torch.cuda.synchronize()
    assert attn.workspace_bytes() > 0 and attn.num_splits() >= 1
    attn.destroy()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))


@pytest.mark.parametrize("wl", [SMALL[0], SMALL[10]], ids=lambda w: w.name)
def test_apply_with_registered_weights(wl):
    x = inputs.make_inputs(wl, seed=18)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    attn = b.CastlingAttn.for_workload(wl)
    o1, o2 = torch.empty_like(t["q"]), torch.empty_like(t["q"])
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], t["w"], None, o1)
    with pytest.raises(b.CastlingError) as e:          # nothing registered yet
        attn.apply(t["q"], t["v"], None, None, o2)
    assert e.value.status == b.ERR_INVALID_ARG
    attn.prepare_weights(t["w"])
    attn.apply(t["q"], t["v"], None, None, o2)
    torch.cuda.synchronize()
    attn.destroy()
    view = torch.int16 if wl.dtype == "bf16" else torch.int32
    assert torch.equal(o1.view(view), o2.view(view))


@pytest.mark.parametrize("wl", [SMALL[10], SMALL[14], SMALL[0]], ids=lambda w: w.name)
def test_registered_weights_survive_other_calls(wl):
    """The operand table of prepare_weights belongs to the registration alone: a backward pass
    (which runs pass 2 with the filters turned by 180 degrees) and a forward with other filters
    in between leave it as it was; forward(w = None) uses it like apply(w = None)."""
    x = inputs.make_inputs(wl, seed=19, with_bias=True)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}
    other_w = (t["w"].float() * -1.7 + 0.05).to(t["w"].dtype)
    attn = b.CastlingAttn.for_workload(wl, flags=b.FLAG_TRAINING)
    o_ref, o_reg, f_ref, f_reg, scratch = (torch.empty_like(t["q"]) for _ in range(5))
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], t["w"], t["bias"], o_ref)
    attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], f_ref)
    with pytest.raises(b.CastlingError) as e:          # nothing registered yet
        attn.forward(t["q"], t["k"], t["v"], None, t["bias"], scratch)
    assert e.value.status == b.ERR_INVALID_ARG
    attn.prepare_weights(t["w"])
    print(f"case registered weights {wl.name}", flush=True)
    grads = [torch.empty_like(t["q"]) for _ in range(3)]
    gw = torch.empty(t["w"].shape, dtype=torch.float32, device=dev)
    attn.backward(t["q"], t["k"], t["v"], other_w, t["v"], grads[0], grads[1], grads[2], gw)
    attn.forward(t["q"], t["k"], t["v"], other_w, t["bias"], scratch)
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], None, t["bias"], o_reg)
    attn.forward(t["q"], t["k"], t["v"], None, t["bias"], f_reg)
    torch.cuda.synchronize()
    attn.destroy()
    view = torch.int16 if wl.dtype != "f32" else torch.int32
    assert torch.equal(o_ref.view(view), o_reg.view(view))
    assert torch.equal(f_ref.view(view), f_reg.view(view))
    assert not torch.equal(scratch.view(view), f_ref.view(view))


@pytest.mark.parametrize("wl", [SMALL[0], SMALL[15], SMALL[10]], ids=lambda w: w.name)
def test_apply_needs_a_reduce(wl):
    """apply() uses what reduce() left in the handle; before any reduce, and after a forward that
    kept its state on chip, there is nothing to apply: an error, not stale data."""
    x = inputs.make_inputs(wl, seed=19)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    attn = b.CastlingAttn.for_workload(wl)
    o = torch.empty_like(t["q"])
    with pytest.raises(b.CastlingError) as e:
        attn.apply(t["q"], t["v"], t["w"], None, o)
    assert e.value.status == b.ERR_INVALID_ARG
    attn.forward(t["q"], t["k"], t["v"], t["w"], None, o)
    if attn.num_launches() == 1:
        with pytest.raises(b.CastlingError) as e:
            attn.apply(t["q"], t["v"], t["w"], None, o)
        assert e.value.status == b.ERR_INVALID_ARG
    attn.reduce(t["k"], t["v"])
    attn.apply(t["q"], t["v"], t["w"], None, o)
    torch.cuda.synchronize()
    attn.destroy()


def test_runs_on_a_side_stream(oracle):
    wl = SMALL[3]
    x = inputs.make_inputs(wl, seed=9)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    out = torch.empty_like(t["q"])
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    attn = b.CastlingAttn.for_workload(wl)
    attn.forward(t["q"], t["k"], t["v"], t["w"], None, out, stream=s)
    s.synchronize()
    attn.destroy()
    q, k, v, w, _ = oracle_inputs(x)
    want = oracle.forward(q, k, v, w, None, wl.grid_h, wl.grid_w)
    assert rel_err(inputs.to_f64(out), want) <= TOL[wl.dtype]


def test_argument_errors_on_device():
    wl = SMALL[0]
    x = inputs.make_inputs(wl)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
    out = torch.empty_like(t["q"])
    attn = b.CastlingAttn.for_workload(wl)
    with pytest.raises(b.CastlingError) as e:
        attn.forward(t["q"], t["k"], t["v"], t["w"], None, t["v"])
    assert e.value.status == b.ERR_ALIAS
    with pytest.raises(b.CastlingError) as e:
        attn.forward(t["q"], t["k"], t["v"], t["w"], None, t["q"])
    assert e.value.status == b.ERR_ALIAS
    with pytest.raises(b.CastlingError) as e:
        attn.forward(None, t["k"], t["v"], t["w"], None, out)
    assert e.value.status == b.ERR_INVALID_ARG
    mis = t["q"].reshape(-1)[1:].clone()           # a fresh buffer, then a view 4 bytes in
    mis_view = torch.empty(t["q"].numel() + 1, dtype=t["q"].dtype, device=dev)[1:]
    with pytest.raises(b.CastlingError) as e:
        attn.forward(mis_view, t["k"], t["v"], t["w"], None, out)
    assert e.value.status == b.ERR_INVALID_ARG
    del mis
    # the handle still works after the refusals
    attn.forward(t["q"], t["k"], t["v"], t["w"], None, out)
    torch.cuda.synchronize()
    attn.destroy()
    assert torch.isfinite(out).all()


@pytest.mark.parametrize("wl", [SMALL[0], SMALL[15], SMALL[10]], ids=lambda w: w.name)
def test_forward_in_a_captured_graph(oracle, wl):
    """forward() only enqueues kernels (no allocation, no synchronisation, no memset), so it can
    be captured in a HIP graph: three-launch fp32 path, one-kernel path, two-pass matrix-core
    path.  Every replay, with eager work and synchronisations in between, must reproduce the
    eager result bit for bit on new inputs written into the captured buffers."""
    dev = torch.device("cuda:0")
    xs = [inputs.make_inputs(wl, seed=60 + i, with_bias=True) for i in range(3)]
    bufs = {n: torch.empty_like(xs[0][n], device=dev) for n in ("q", "k", "v", "w", "bias")}
    out = torch.empty_like(bufs["q"])
    eager_out = torch.empty_like(bufs["q"])
    attn = b.CastlingAttn.for_workload(wl)
    side = torch.cuda.Stream()
    for n in bufs:
        bufs[n].copy_(xs[0][n])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        attn.forward(bufs["q"], bufs["k"], bufs["v"], bufs["w"], bufs["bias"], out, stream=side)  # warm-up
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            attn.forward(bufs["q"], bufs["k"], bufs["v"], bufs["w"], bufs["bias"], out,
                         stream=torch.cuda.current_stream())
    for i, x in enumerate(xs):
        print(f"case graph replay {wl.name} #{i}", flush=True)
        for n in bufs:
            bufs[n].copy_(x[n])
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        attn.forward(bufs["q"], bufs["k"], bufs["v"], bufs["w"], bufs["bias"], eager_out)
        torch.cuda.synchronize()
        view = torch.int32 if wl.dtype == "f32" else torch.int16
        assert torch.equal(out.view(view), eager_out.view(view))
        q, k, v, w, bias = oracle_inputs(x)
        want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
        assert rel_err(inputs.to_f64(out), want) <= TOL[wl.dtype]
    del graph
    attn.destroy()


def test_two_handles_on_two_streams(oracle):
    """Handles are independent: forwards of two handles (different shapes and paths) enqueued
    alternately on two streams give the same bits as each handle run alone."""
    dev = torch.device("cuda:0")
    wls = [SMALL[10], SMALL[15]]                      # two-pass matrix-core path, one-kernel path
    xs = [inputs.make_inputs(wl, seed=70 + i, with_bias=True) for i, wl in enumerate(wls)]
    ts = [{n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")} for x in xs]
    handles = [b.CastlingAttn.for_workload(wl) for wl in wls]
    alone = []
    for h, t in zip(handles, ts):
        o = torch.empty_like(t["q"])
        h.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], o)
        torch.cuda.synchronize()
        alone.append(o)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.empty_like(t["q"]) for t in ts]
    torch.cuda.synchronize()
    for _ in range(20):
        for h, t, o, s in zip(handles, ts, outs, streams):
            h.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], o, stream=s)
    for s in streams:
        s.synchronize()
    for h in handles:
        h.destroy()
    for o, a, wl, x in zip(outs, alone, wls, xs):
        assert torch.equal(o.view(torch.int16), a.view(torch.int16))
        q, k, v, w, bias = oracle_inputs(x)
        want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
        assert rel_err(inputs.to_f64(o), want) <= TOL[wl.dtype]


@pytest.mark.parametrize("dtype,C_,ks", [("bf16", 256, 3), ("f16", 384, 5), ("f32", 128, 3)])
def test_dwconv_on_token_major_features(oracle, dtype, C_, ks):
    """The DWConv branch alone on a token-major [B][N][C] tensor (the depthwise convolution the
    paper also places between the two MLP layers, Sec. 4.3): C channels as C / 64 heads of 64,
    input and output with (batch, head, token) strides (N C, 64, C)."""
    B, H, W, d = 2, 12, 20, 64
    heads, N = C_ // d, H * W
    wl = Workload(f"mlp_{dtype}_c{C_}", dtype, B, heads, d, H, W, ks)
    x = inputs.make_inputs(wl, seed=53, with_bias=True)
    dev = torch.device("cuda:0")
    feat = x["v"].to(dev).permute(0, 2, 1, 3).reshape(B, N, C_).contiguous()
    out = torch.full_like(feat, float("nan"))
    tm = b.token_major_strides(heads, N, d)
    attn = b.CastlingAttn.for_workload(wl, branches=b.BRANCH_DWCONV, in_strides=tm, out_strides=tm)
    attn.forward(feat, feat, feat, x["w"].to(dev), x["bias"].to(dev), out)
    torch.cuda.synchronize()
    attn.destroy()
    q, k, v, w, bias = oracle_inputs(x)
    want = oracle.forward(q, k, v, w, bias, H, W, branches=b.BRANCH_DWCONV)
    got = inputs.to_f64(out.view(B, N, heads, d).permute(0, 2, 1, 3))
    assert rel_err(got, want) <= TOL[dtype]


@pytest.mark.parametrize("wl", HEAD_PAIRS, ids=lambda w: w.name)
@pytest.mark.parametrize("norm", [b.NORM_ROWSUM, b.NORM_NONE])
def test_pairs_of_narrow_heads(oracle, wl, norm):
    x = inputs.make_inputs(wl, seed=61, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    for branches in (b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV):
        print(f"case {wl.name} norm={norm} branches={branches}", flush=True)
        want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w, norm=norm, branches=branches)
        if branches & b.BRANCH_LINEAR:
            got, st = gpu_forward(wl, x, norm=norm, branches=branches, want_state=True)
            assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]
        else:
            got = gpu_forward(wl, x, norm=norm, branches=branches)
        assert rel_err(got, want) <= TOL[wl.dtype], (wl.name, norm, branches)
        strided = gpu_forward_fused(wl, x, norm=norm, branches=branches)
        assert rel_err(strided, want) <= TOL[wl.dtype], (wl.name, norm, branches, "fused layout")
        # head rows of 40 elements: the two halves of a pair's token row are not adjacent
        padded = gpu_forward_fused(wl, x, norm=norm, branches=branches, pad=8)
        assert rel_err(padded, want) <= TOL[wl.dtype], (wl.name, norm, branches, "padded heads")


def test_pairs_of_narrow_heads_take_the_matrix_core_path():
    """Launch counts tell the paths apart.  Small units: one kernel for pairs, two launches on the
    vector-ALU path an odd head count is left with.  Large units with one split each: the
    vector-ALU path needs two launches, the pair path three (its operand tables come from a
    combine launch of their own)."""
    def launches(wl, **kw):
        h = b.CastlingAttn.for_workload(wl, **kw)
        n, s = h.num_launches(), h.num_splits()
        h.destroy()
        return n, s
    assert launches(HEAD_PAIRS[4]) == (1, 1)
    assert launches(Workload("hp_odd", "bf16", 32, 9, 32, 7, 7, 3)) == (2, 1)
    assert launches(Workload("hp_big", "bf16", 32, 8, 32, 20, 20, 3)) == (3, 1)
    assert launches(Workload("hp_big_odd", "bf16", 32, 9, 32, 20, 20, 3)) == (2, 1)
    assert launches(HEAD_PAIRS[4], flags=b.FLAG_SEPARATE_PASSES) == (3, 1)


@pytest.mark.parametrize("wl", [
    Workload("one_unit_bf16_512x768_k5", "bf16", 1, 1, 64, 512, 768, 5),
    Workload("one_unit_f32_d32_256x256_k3", "f32", 1, 1, 32, 256, 256, 3),
    Workload("two_units_f16_d32_384x256_k7", "f16", 1, 2, 32, 384, 256, 7),
], ids=lambda w: w.name)
def test_one_unit_with_the_maximum_number_of_splits(oracle, wl):
    """A single long unit: pass 1 splits it over every compute unit (256 partial states per unit,
    summed in index order), pass 2 hands every block a stretch of one and the same unit."""
    x = inputs.make_inputs(wl, seed=71, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    h = b.CastlingAttn.for_workload(wl)
    splits = h.num_splits()
    h.destroy()
    assert splits >= 128
    got, st = gpu_forward(wl, x, want_state=True)
    assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]
    assert rel_err(got, want) <= TOL[wl.dtype]
