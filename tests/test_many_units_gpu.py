"""Whole-layer parity on shapes with many units (hundreds of batch x head pairs of a few hundred
to a few thousand tokens), where every workgroup of the persistent pass-2 kernel walks through
several units and the pass-1 grid is several times the chip.  Two runs must agree bitwise."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import TOL, STATE_TOL, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# units x tiles far above the number of resident workgroups
MANY_TASKS = [
    Workload("st_bf16_b128_h8_12x24_k3", "bf16", 128, 8, 64, 12, 24, 3),    # 1024 units
    Workload("st_f16_b64_h8_16x40_k5", "f16", 64, 8, 64, 16, 40, 5),        # 512 units
    Workload("st_bf16_b40_h6_27x28_k3", "bf16", 40, 6, 64, 27, 28, 3),      # 240 units, ragged strips
    Workload("st_bf16_b32_h8_32x32_k5", "bf16", 32, 8, 64, 32, 32, 5),      # 256 units, 2 reduce chunks + combine
]
# Shapes written for an experimental one-kernel form of the whole forward (pass 1, the sum of
# its partial states and pass 2 as tasks of one persistent kernel).  The first ran correctly
# there; the second (24 units of 8000 tokens, 7 x 7 filters) faulted the GPU in that kernel, as
# the largest benchmark workload did, and the cause was not found.  That kernel is no longer part
# of the library; the cases stay, skipped, as the record of what it was run on.
MANY_CHUNKS = [
    Workload("st_f16_b8_h8_48x48_k9", "f16", 8, 8, 64, 48, 48, 9),          # 64 units, 4 reduce chunks
    Workload("st_bf16_b4_h6_40x200_k7", "bf16", 4, 6, 64, 40, 200, 7),      # 24 units (3 per queue), 16 chunks each
]


@pytest.mark.skip(reason="cases of the removed one-kernel forward, which faulted the GPU on long units "
                         "(cause not found); kept as its record")
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
    outs = []
    for rep in range(2):
        out = torch.full_like(t["q"], float("nan"))
        attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], out)
        torch.cuda.synchronize()
        outs.append(out)
    st = attn.get_state()
    attn.destroy()
    want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w)
    assert rel_err(inputs.to_f64(outs[0]), want) <= TOL[wl.dtype]
    assert rel_err(st, oracle.state(k, v)) <= STATE_TOL[wl.dtype]
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
