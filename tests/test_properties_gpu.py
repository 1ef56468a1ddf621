"""Property-based GPU parity (hypothesis, a fixed derandomised set of examples): the HIP layer
through the C ABI against the oracle's explicit N x N definition on small random shapes, over
every I/O type, head width the kernels accept, filter size, branch set, normaliser mode and
number of class tokens."""
import numpy as np
import pytest
import torch
from hypothesis import HealthCheck, given, settings
from hypothesis import strategies as st

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import TOL, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

SETTINGS = dict(max_examples=40, deadline=None, derandomize=True,
                suppress_health_check=[HealthCheck.function_scoped_fixture, HealthCheck.too_slow])


@st.composite
def shapes(draw):
    dtype = draw(st.sampled_from(["bf16", "f16", "f32"]))
    d = draw(st.sampled_from([8, 16, 24, 32, 64, 96, 128]))
    B = draw(st.integers(1, 3))
    heads = draw(st.integers(1, 4))
    H = draw(st.integers(1, 20))
    W = draw(st.integers(1, 20))
    ks = draw(st.sampled_from([1, 3, 5, 7, 9]))
    extra = draw(st.integers(0, 2))
    norm = draw(st.sampled_from([b.NORM_ROWSUM, b.NORM_NONE]))
    branches = draw(st.sampled_from([b.BRANCH_ALL, b.BRANCH_LINEAR, b.BRANCH_DWCONV]))
    seed = draw(st.integers(0, 10 ** 6))
    return dtype, B, heads, d, H, W, ks, extra, norm, branches, seed


@settings(**SETTINGS)
@given(case=shapes())
def test_forward_equals_the_definition_on_random_shapes(oracle, case):
    dtype, B, heads, d, H, W, ks, extra, norm, branches, seed = case
    wl = Workload("prop", dtype, B, heads, d, H, W, ks)
    flat = Workload("prop", dtype, B, heads, d, 1, wl.N + extra, ks)   # inputs for N + extra tokens
    x = inputs.make_inputs(flat, seed=seed, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    print(f"case property {case}", flush=True)
    want = oracle.forward_explicit(q, k, v, w, bias, H, W, norm=norm, branches=branches, extra=extra)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}
    out = torch.full_like(t["q"], float("nan"))
    attn = b.CastlingAttn.for_workload(wl, norm=norm, branches=branches, extra_tokens=extra)
    attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], out)
    torch.cuda.synchronize()
    attn.destroy()
    got = inputs.to_f64(out)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL[dtype], case
