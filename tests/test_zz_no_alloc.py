"""castling_attn_forward_static (the forward that allocates nothing: its workspace is a fixed
array inside the library's device image) against castling_attn_forward on a handle, through the
C ABI.  The same kernels run on both sides, so the outputs must agree bitwise; two calls in a row
share the array, the second with a smaller problem of another layout."""
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload

pytestmark = pytest.mark.gpu

# (first, second): the second call is the smaller problem and lays the array out differently
SEQUENCES = [
    # two-pass matrix-core path with several token splits, then the one-kernel path
    (Workload("na_bf16_b2_h3_40x72_k3", "bf16", 2, 3, 64, 40, 72, 3),
     Workload("na_bf16_b1_h2_14x14_k3", "bf16", 1, 2, 64, 14, 14, 3)),
    # fp16 two-pass, then a smaller two-pass shape with another filter size
    (Workload("na_f16_b2_h4_33x40_k5", "f16", 2, 4, 64, 33, 40, 5),
     Workload("na_f16_b1_h3_20x36_k7", "f16", 1, 3, 64, 20, 36, 7)),
    # vector-ALU kernels (fp32), then pairs of 32-channel heads on the matrix cores
    (Workload("na_f32_b2_h4_d32_20x24_k3", "f32", 2, 4, 32, 20, 24, 3),
     Workload("na_bf16_b1_h4_d32_14x14_k5", "bf16", 1, 4, 32, 14, 14, 5)),
]


def _desc(wl, flags=0):
    return b.make_desc(wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype,
                       flags=flags)


def _device_inputs(wl, seed):
    x = inputs.make_inputs(wl, seed=seed, with_bias=True)
    dev = torch.device("cuda:0")
    return {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}


def _bits(t):
    return t.view(torch.int32 if t.element_size() == 4 else torch.int16)


@pytest.mark.parametrize("first,second", SEQUENCES, ids=lambda w: w.name)
def test_static_scratch_forward_equals_handle_forward(first, second):
    for i, wl in enumerate((first, second)):
        t = _device_inputs(wl, seed=70 + i)
        attn = b.CastlingAttn.for_workload(wl)
        assert attn.workspace_bytes() <= b.STATIC_SCRATCH_BYTES
        want = torch.full_like(t["q"], float("nan"))
        attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], want)
        torch.cuda.synchronize()
        attn.destroy()
        print(f"case static scratch {wl.name} (call {i + 1} of 2)", flush=True)
        got = torch.full_like(t["q"], float("nan"))
        b.forward_static(_desc(wl), t["q"], t["k"], t["v"], t["w"], t["bias"], got)
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        assert torch.equal(_bits(got), _bits(want)), wl.name


def test_static_scratch_forward_refuses_what_does_not_fit():
    big = Workload("na_big", "bf16", 128, 8, 64, 12, 24, 3)      # 1024 units: 2 x 17 MB of states and the operand tables
    t = _device_inputs(Workload("na_tiny", "bf16", 1, 1, 64, 4, 4, 3), seed=72)
    out = torch.empty_like(t["q"])
    with pytest.raises(b.CastlingError) as e:                    # refused before any pointer is used
        b.forward_static(_desc(big), t["q"], t["k"], t["v"], t["w"], t["bias"], out)
    assert e.value.status == b.ERR_TOO_LARGE
    assert "scratch" in str(e.value)
    with pytest.raises(b.CastlingError) as e:
        b.forward_static(_desc(big, flags=b.FLAG_TRAINING), t["q"], t["k"], t["v"], t["w"], t["bias"], out)
    assert e.value.status == b.ERR_INVALID_ARG
    small = Workload("na_tiny", "bf16", 1, 1, 64, 4, 4, 3)
    with pytest.raises(b.CastlingError) as e:                    # no registration to fall back on
        b.forward_static(_desc(small), t["q"], t["k"], t["v"], None, t["bias"], out)
    assert e.value.status == b.ERR_INVALID_ARG


def test_benchmark_workloads_fit_the_static_scratch():
    sizes = {}
    for wl in inputs.WORKLOADS:
        attn = b.CastlingAttn.for_workload(wl)
        sizes[wl.name] = attn.workspace_bytes()
        attn.destroy()
    print("workspace bytes:", sizes, flush=True)
    assert max(sizes.values()) <= b.STATIC_SCRATCH_BYTES
