"""The one-launch forward (pass 1, combine and pass 2 as tasks of one persistent kernel) on shapes
where every workgroup runs several tasks of different kinds one after the other, against the
oracle; the in-kernel checks must stay silent."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import TOL, STATE_TOL, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# units x (reduce task + apply chunks) far above the 512 resident workgroups
MANY_TASKS = [
    Workload("st_bf16_b128_h8_12x24_k3", "bf16", 128, 8, 64, 12, 24, 3),    # 1024 units
    Workload("st_f16_b64_h8_16x40_k5", "f16", 64, 8, 64, 16, 40, 5),        # 512 units
    Workload("st_bf16_b40_h6_27x28_k3", "bf16", 40, 6, 64, 27, 28, 3),      # 240 units, ragged strips
]
# Units of several reduce chunks: the first two ran correctly through the one-launch forward,
# the third (24 units of 8000 tokens, 16 chunks each) faulted the GPU, as the largest benchmark
# workload (24 units of 16384 tokens) did; the cause is not known.  The library now keeps such
# shapes on the separate launches (castling_attn.hip, plan_stream), so these cases no longer
# reach the kernel they were written for.
MANY_CHUNKS = [
    Workload("st_bf16_b32_h8_32x32_k5", "bf16", 32, 8, 64, 32, 32, 5),      # 256 units, 2 reduce chunks + combine
    Workload("st_f16_b8_h8_48x48_k9", "f16", 8, 8, 64, 48, 48, 9),          # 64 units, 4 reduce chunks
    Workload("st_bf16_b4_h6_40x200_k7", "bf16", 4, 6, 64, 40, 200, 7),      # 24 units (3 per queue), 16 chunks each
]


@pytest.mark.skip(reason="one-launch forward with several reduce chunks per unit: faulted the GPU at 16 "
                         "chunks per unit, cause unknown; the code path is switched off in plan_stream")
@pytest.mark.parametrize("wl", MANY_CHUNKS, ids=lambda w: w.name)
def test_many_chunks_per_unit(oracle, wl):
    test_many_tasks_per_workgroup(oracle, wl)


@pytest.mark.parametrize("wl", MANY_TASKS, ids=lambda w: w.name)
def test_many_tasks_per_workgroup(oracle, wl):
    x = inputs.make_inputs(wl, seed=31, with_bias=True)
    q, k, v, w, bias = oracle_inputs(x)
    dev = torch.device("cuda:0")
    t = {n: x[n].to(dev) for n in ("q", "k", "v", "w", "bias")}
    print(f"case many tasks {wl.name}: q {t['q'].data_ptr():#x} k {t['k'].data_ptr():#x} "
          f"v {t['v'].data_ptr():#x}", flush=True)
    attn = b.CastlingAttn.for_workload(wl, flags=b.FLAG_KEEP_STATE)
    assert attn.num_launches() == 1
    outs = []
    for rep in range(2):
        out = torch.full_like(t["q"], float("nan"))
        attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], out)
        attn.check()
        outs.append(out)
    st = attn.get_state()
    attn.destroy()
    want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    assert rel_err(inputs.to_f64(outs[0]), want) <= TOL[wl.dtype]
    assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
