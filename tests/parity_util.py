"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch

from paper_2211_10526_amd import binding as b
from paper_2211_10526_amd import inputs

# fp16 I/O (fp32 products and accumulation): the output rounding, 2^-11 = 4.9e-4 relative,
# dominates; 1e-3 leaves a factor of two
TOL = {"f32": 1e-4, "bf16": 1e-2, "f16": 1e-3}
# The exported state K_hat^T V: the matrix-core kernels round k_hat to the I/O format before
# the contraction, so every product carries up to half an ulp (2^-11 for fp16) of relative
# error; against rms(S) that is about 2^-11 / sqrt(3) per element and about 4.5 times as much
# at the maximum over 10^6 elements: 1.3e-3 for fp16 (bf16, 8 times coarser, stays inside its
# 1e-2).  The state is an intermediate, not an output of the layer.
STATE_TOL = {"f32": 1e-4, "bf16": 1e-2, "f16": 2.5e-3}

# Gradients: the forward output is dominated by exactly accumulated terms (vsum / 2, the
# convolution) with the state-dependent part a correction; a gradient with respect to q or k is
# linear in the state K_hat^T V (or Q_hat^T a) throughout, so it inherits the state's error
# (k_hat, and a = g / den, rounded to the I/O type before the contraction) on top of its own
# output rounding: two to three roundings of 2^-9 (bf16) in a row, about 4.5 standard deviations
# at the maximum over 10^5 .. 10^6 elements.  fp32 I/O keeps fp32 products: the forward's bound.
GRAD_TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2.5e-3}


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |g_i - o_i| / max(|o_i|, rms(o)): the layer's parity metric."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    rms = float(np.sqrt(np.mean(want * want)))
    if rms == 0.0:
        return float(np.max(np.abs(got - want)))
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), rms)))


def gpu_forward(wl, x, norm=b.NORM_ROWSUM, branches=b.BRANCH_ALL, eps=0.0, want_state=False, flags=0):
    """Runs the HIP layer through the C ABI; returns float64 numpy [B,heads,N,d]."""
    dev = torch.device("cuda:0")
    t = {n: (None if x[n] is None else x[n].to(dev)) for n in ("q", "k", "v", "w", "bias")}
    out = torch.empty_like(t["q"])
    out.fill_(float("nan"))
    attn = b.CastlingAttn.for_workload(wl, norm=norm, branches=branches, eps=eps,
                                       flags=flags | (b.FLAG_KEEP_STATE if want_state else 0))
    attn.forward(t["q"], t["k"], t["v"], t["w"], t["bias"], out)
    torch.cuda.synchronize()
    res = inputs.to_f64(out)
    st = attn.get_state() if want_state else None
    attn.destroy()
    return (res, st) if want_state else res


def gpu_forward_fused(wl, x, norm=b.NORM_ROWSUM, branches=b.BRANCH_ALL, eps=0.0, want_state=False,
                      pad=0):
    """As gpu_forward, with projection-adjacent layouts: q, k, v are the slices of one fused
    [B][N][3][heads][d (+ pad)] tensor and out is [B][N][heads * d].  Only data movement
    happens here; the result comes back as float64 [B,heads,N,d]."""
    dev = torch.device("cuda:0")
    B, H, N, d = wl.B, wl.heads, wl.N, wl.d
    dp = d + pad
    qkv = torch.full((B, N, 3, H, dp), float("nan"), dtype=x["q"].dtype, device=dev)
    for i, n in enumerate(("q", "k", "v")):
        qkv[:, :, i, :, :d] = x[n].to(dev).permute(0, 2, 1, 3)  # [B,H,N,d] -> [B,N,H,d]
    q, k, v = (qkv[:, :, i, :, :d] for i in range(3))
    w = x["w"].to(dev)
    bias = None if x["bias"] is None else x["bias"].to(dev)
    out = torch.full((B, N, H * d), float("nan"), dtype=x["q"].dtype, device=dev)
    attn = b.CastlingAttn.for_workload(
        wl, norm=norm, branches=branches, eps=eps,
        in_strides=(N * 3 * H * dp, dp, 3 * H * dp), out_strides=b.token_major_strides(H, N, d),
        flags=b.FLAG_KEEP_STATE if want_state else 0)
    attn.forward(q, k, v, w, bias, out)
    torch.cuda.synchronize()
    res = inputs.to_f64(out.view(B, N, H, d).permute(0, 2, 1, 3).contiguous())
    st = attn.get_state() if want_state else None
    attn.destroy()
    return (res, st) if want_state else res


def oracle_inputs(x):
    return tuple(inputs.to_f64(x[n]) for n in ("q", "k", "v", "w", "bias"))
