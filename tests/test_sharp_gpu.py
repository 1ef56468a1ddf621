"""16-bit parity where the attention-specific terms are the whole signal.

On iid Gaussian inputs the output of the linear branch is dominated by mean(V); the terms that
make the method what it is (q_hat . K_hat^T V / pi in the numerator, q_hat . sum_j k_hat_j / pi
in the normaliser; Eq. 3 and the linear terms of Eq. 8) are corrections of a few percent there.
These inputs remove that cover, on the one-kernel path, on the two-pass matrix-core path at
the same shape, and on a two-pass shape with several strips and token splits per unit:

  zero column sums of V, no normaliser: the output *is* q_hat . S / pi;
  all keys equal, V constant per channel: every weight is the same, the output is the constant
      (to output rounding) whatever the query - any inconsistency between the numerator's
      tables and the normaliser's shows;
  keys and queries around one common direction: q_hat . ksum / pi is about a third of the
      normaliser instead of a few percent.

Each against the oracle element by element."""
import numpy as np
import pytest
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs
from paper_2211_10526_amd.inputs import Workload
from parity_util import TOL, gpu_forward, oracle_inputs, rel_err

pytestmark = pytest.mark.gpu

# (workload, flags): N = 196 in one kernel and as reduce + apply; 2880 tokens per unit in
# two 64-column strips with several token splits in pass 1
CASES = [
    (Workload("sh_bf16_14x14_k3", "bf16", 2, 3, 64, 14, 14, 3), 0),
    (Workload("sh_bf16_14x14_k3", "bf16", 2, 3, 64, 14, 14, 3), b.FLAG_SEPARATE_PASSES),
    (Workload("sh_f16_14x14_k5", "f16", 2, 3, 64, 14, 14, 5), 0),
    (Workload("sh_f16_14x14_k5", "f16", 2, 3, 64, 14, 14, 5), b.FLAG_SEPARATE_PASSES),
    (Workload("sh_bf16_40x72_k3", "bf16", 1, 4, 64, 40, 72, 3), 0),
    (Workload("sh_f16_40x72_k3", "f16", 1, 4, 64, 40, 72, 3), 0),
]
IDS = [f"{wl.name}{'_two_pass' if fl else ''}" for wl, fl in CASES]
# unit roundoff of the stored type
ROUNDOFF = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}
# Where the state term is the whole output nothing exactly accumulated dilutes its error: the
# matrix-core paths round q_hat and the state table to the stored type, so every one of the d
# products carries two roundings (each about 0.4 unit roundoffs rms); their sum has that
# relative error against the output's rms (random signs on both), about 0.6 roundoffs rms and
# 4.5 times as much at the maximum over 10^5 .. 10^6 elements, plus the output's own rounding
# of up to one roundoff: 1.4e-2 for bf16, 1.8e-3 for fp16.  The bounds below leave a third on
# top; a systematic error of 3 % in the term fails them.
STATE_TERM_TOL = {"bf16": 2e-2, "f16": 2.5e-3}


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


@pytest.mark.parametrize("wl,flags", CASES, ids=IDS)
def test_output_is_the_state_term_alone(oracle, wl, flags):
    """V in antisymmetric halves: its column sums are exactly zero in the stored type, so
    without the normaliser out_t = q_hat_t . (K_hat^T V) / pi and nothing else."""
    x = inputs.make_inputs(wl, seed=41)
    half = wl.N // 2
    assert wl.N == 2 * half
    x["v"][:, :, half:] = -x["v"][:, :, :half]
    q, k, v, w, bias = oracle_inputs(x)
    assert np.all(v.sum(axis=2) == 0.0)
    print(f"case state term alone {wl.name} flags={flags}", flush=True)
    got = gpu_forward(wl, x, norm=b.NORM_NONE, branches=b.BRANCH_LINEAR, flags=flags)
    want = oracle.forward(q, k, v, w, None, wl.grid_h, wl.grid_w, norm=b.NORM_NONE,
                          branches=b.BRANCH_LINEAR)
    assert np.isfinite(got).all()
    # the signal is not small against what the usual inputs give: O(sqrt(N)) per element
    assert np.sqrt(np.mean(want * want)) > 0.1
    assert rel_err(got, want) <= STATE_TERM_TOL[wl.dtype]
    # no systematic factor on the term: the least-squares scale of got against want is 1
    scale = float(np.sum(got * want) / np.sum(want * want))
    assert abs(scale - 1.0) <= 0.1 * STATE_TERM_TOL[wl.dtype], scale


@pytest.mark.parametrize("wl,flags", CASES, ids=IDS)
@pytest.mark.parametrize("aligned", [False, True], ids=["random_queries", "aligned_queries"])
def test_equal_keys_and_constant_v_give_the_constant(oracle, wl, flags, aligned):
    """All keys equal: A_tj does not depend on j, so the normalised output is the mean of V,
    and with V constant per channel that is the constant itself.  With the queries near the
    keys' direction the q_hat . ksum / pi part of the normaliser is at its largest (about 0.3
    against the 0.5 of the constant term)."""
    x = inputs.make_inputs(wl, seed=42)
    g = _gen(43)
    dt = x["q"].dtype
    k0 = torch.randn((wl.B, wl.heads, 1, wl.d), generator=g)
    x["k"] = k0.expand(-1, -1, wl.N, -1).to(dt).contiguous()
    if aligned:
        x["q"] = (k0 * 1.5 + 0.3 * torch.randn((wl.B, wl.heads, wl.N, wl.d), generator=g)).to(dt).contiguous()
    c = torch.randn((wl.B, wl.heads, 1, wl.d), generator=g).to(dt)
    x["v"] = c.expand(-1, -1, wl.N, -1).contiguous()
    q, k, v, w, bias = oracle_inputs(x)
    print(f"case equal keys {wl.name} flags={flags} aligned={aligned}", flush=True)
    got = gpu_forward(wl, x, branches=b.BRANCH_LINEAR, flags=flags)
    want = oracle.forward(q, k, v, w, None, wl.grid_h, wl.grid_w, branches=b.BRANCH_LINEAR)
    np.testing.assert_allclose(want, np.broadcast_to(v[:, :, :1], want.shape), rtol=1e-12, atol=0)
    if aligned:
        qh = q / np.linalg.norm(q, axis=-1, keepdims=True)
        kh = k[:, :, :1] / np.linalg.norm(k[:, :, :1], axis=-1, keepdims=True)
        assert np.mean(np.sum(qh * kh, axis=-1)) / np.pi > 0.25
    # the constant to output rounding: two unit roundoffs of the stored type, relative per element
    err = np.max(np.abs(got - want) / np.abs(want).clip(min=np.sqrt(np.mean(want * want))))
    assert err <= 2.0 * ROUNDOFF[wl.dtype], err
    assert np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-3)) <= 4.0 * ROUNDOFF[wl.dtype]


@pytest.mark.parametrize("wl,flags", CASES, ids=IDS)
@pytest.mark.parametrize("branches", [b.BRANCH_LINEAR, b.BRANCH_ALL], ids=["linear", "all"])
def test_keys_aligned_with_the_queries(oracle, wl, flags, branches):
    """Keys and queries scattered around one direction per unit: every similarity is far from
    1/2, the normaliser's state-dependent part is about a third of it, and the weights vary
    over the keys, so V's structure shows through the state term."""
    x = inputs.make_inputs(wl, seed=44, with_bias=True)
    g = _gen(45)
    dt = x["q"].dtype
    axis = torch.randn((wl.B, wl.heads, 1, wl.d), generator=g)
    x["q"] = (axis + 0.5 * torch.randn((wl.B, wl.heads, wl.N, wl.d), generator=g)).to(dt).contiguous()
    x["k"] = (axis + 0.5 * torch.randn((wl.B, wl.heads, wl.N, wl.d), generator=g)).to(dt).contiguous()
    q, k, v, w, bias = oracle_inputs(x)
    qh = q / np.linalg.norm(q, axis=-1, keepdims=True)
    kh = k / np.linalg.norm(k, axis=-1, keepdims=True)
    lin_part = np.einsum("bhnd,bhd->bhn", qh, kh.mean(axis=2)) / np.pi
    assert lin_part.mean() > 0.2          # against 0.5: the normaliser is not mostly the constant
    print(f"case aligned keys {wl.name} flags={flags} branches={branches}", flush=True)
    for norm in (b.NORM_ROWSUM, b.NORM_NONE):
        got = gpu_forward(wl, x, norm=norm, branches=branches, flags=flags)
        want = oracle.forward(q, k, v, w, bias, wl.grid_h, wl.grid_w, norm=norm, branches=branches)
        assert rel_err(got, want) <= TOL[wl.dtype], norm
