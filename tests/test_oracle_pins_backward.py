"""Pins of the oracle's backward pass against things other than itself: torch autograd through
a plain torch (fp64) transcription of the forward definition (Eq. 3, 8, 9), central finite
differences of the oracle's own, separately pinned, forward, and structural facts (the
gradient of a constant value row, the tangent-space property of the normalisation)."""
import math

import numpy as np
import pytest
import torch

PI = math.pi


def draw(seed, B, heads, H, W, d, ks, extra=0):
    r = np.random.default_rng(seed)
    N = extra + H * W
    q, k, v, g = (r.normal(size=(B, heads, N, d)) for _ in range(4))
    w = r.normal(size=(heads, d, ks, ks)) * 0.3
    bias = r.normal(size=(heads, d))
    return q, k, v, w, bias, g


def torch_forward(q, k, v, w, bias, H, W, norm, branches, eps, extra, residual):
    """The layer in plain torch ops, as Eq. 9 reads with the oracle's readings."""
    B, heads, N, d = q.shape
    out = torch.zeros_like(q)
    if branches & 1:
        qh = q / torch.clamp(q.norm(dim=-1, keepdim=True), min=eps)
        kh = k / torch.clamp(k.norm(dim=-1, keepdim=True), min=eps)
        A = 0.5 + qh @ kh.transpose(-1, -2) / PI
        lin = A @ v
        if norm == 0:
            lin = lin / A.sum(-1, keepdim=True)
        out = out + lin
    if branches & 2:
        ks = w.shape[-1]
        x = v[:, :, extra:].reshape(B, heads, H, W, d).permute(0, 1, 4, 2, 3).reshape(B, heads * d, H, W)
        y = torch.nn.functional.conv2d(x, w.reshape(heads * d, 1, ks, ks), bias.reshape(-1),
                                       padding=ks // 2, groups=heads * d)
        y = y.reshape(B, heads, d, H, W).permute(0, 1, 3, 4, 2).reshape(B, heads, H * W, d)
        out = torch.cat([out[:, :, :extra], out[:, :, extra:] + y], dim=2)
    if residual:
        out = out + q
    return out


CASES = [
    # B, heads, H, W, d, ks, extra
    (2, 2, 4, 5, 6, 3, 0),
    (1, 3, 3, 7, 4, 5, 1),
    (1, 1, 6, 6, 8, 1, 0),
    (2, 1, 2, 9, 3, 7, 2),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("norm", [0, 1])
@pytest.mark.parametrize("branches", [3, 1, 2])
def test_gradients_equal_autograd_of_the_definition(oracle, case, norm, branches):
    B, heads, H, W, d, ks, extra = case
    q, k, v, w, bias, g = draw(81, *case)
    # a floor of the norm that some rows fall under: both branches of the normalisation
    eps = 0.9 * math.sqrt(d)
    residual = branches & 1
    tq, tk, tv, tw, tb = (torch.tensor(a, requires_grad=True) for a in (q, k, v, w, bias))
    out = torch_forward(tq, tk, tv, tw, tb, H, W, norm, branches, eps, extra, residual)
    np.testing.assert_allclose(
        out.detach().numpy() - (q if residual else 0),
        oracle.forward_explicit(q, k, v, w, bias, H, W, norm=norm, branches=branches, eps=eps,
                                extra=extra), atol=1e-12)
    (out * torch.tensor(g)).sum().backward()
    want = [t.grad.numpy() if t.grad is not None else np.zeros(t.shape) for t in (tq, tk, tv, tw, tb)]
    small = (np.linalg.norm(q, axis=-1) < eps).mean()
    assert 0.1 < small < 0.9
    for fn in (oracle.backward_explicit, oracle.backward):
        got = fn(q, k, v, w, g, H, W, norm=norm, branches=branches, eps=eps, extra=extra,
                 residual=residual)
        for name, a, b in zip(("dq", "dk", "dv", "dw", "dbias"), got, want):
            np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-10, err_msg=f"{fn.__name__} {name}")


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("norm", [0, 1])
@pytest.mark.parametrize("branches", [3, 1, 2])
def test_sampled_gradient_rows_equal_autograd_of_the_definition(oracle, case, norm, branches):
    """backward_explicit_rows (the full-size check of the kernels' gradients) on every token of
    every unit, asked for in a scrambled order, against autograd through the plain torch forward."""
    B, heads, H, W, d, ks, extra = case
    q, k, v, w, bias, g = draw(85, *case)
    eps = 0.9 * math.sqrt(d)
    residual = branches & 1
    tq, tk, tv, tw, tb = (torch.tensor(a, requires_grad=True) for a in (q, k, v, w, bias))
    out = torch_forward(tq, tk, tv, tw, tb, H, W, norm, branches, eps, extra, residual)
    (out * torch.tensor(g)).sum().backward()
    want = [t.grad.numpy() if t.grad is not None else np.zeros(t.shape) for t in (tq, tk, tv)]
    N = extra + H * W
    r = np.random.default_rng(5)
    pick = r.permutation(B * heads * N)
    units, tokens = pick // N, pick % N
    got = oracle.backward_explicit_rows(q, k, v, w, g, H, W, units, tokens, norm=norm,
                                        branches=branches, eps=eps, extra=extra, residual=residual)
    for name, a, b in zip(("dq", "dk", "dv"), got, want):
        np.testing.assert_allclose(a, b.reshape(B * heads, N, d)[units, tokens], rtol=1e-9, atol=1e-10,
                                   err_msg=name)


def test_sampled_gradient_rows_at_a_larger_size(oracle):
    """A few rows of two units against the full explicit backward (itself pinned above), on a
    shape where the filter is wider than the grid's short side."""
    case = (1, 3, 4, 33, 16, 9, 2)
    B, heads, H, W, d, ks, extra = case
    q, k, v, w, bias, g = draw(86, *case)
    N = extra + H * W
    units = np.array([2, 0, 2, 0, 2, 0])
    tokens = np.array([0, 1, N - 1, extra, extra + W, 57])
    for norm in (0, 1):
        full = oracle.backward_explicit(q, k, v, w, g, H, W, norm=norm, extra=extra)
        rows = oracle.backward_explicit_rows(q, k, v, w, g, H, W, units, tokens, norm=norm, extra=extra)
        for a, b in zip(rows, full[:3]):
            np.testing.assert_allclose(a, b.reshape(B * heads, N, d)[units, tokens], rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("case", CASES[:2])
@pytest.mark.parametrize("norm", [0, 1])
def test_directional_derivatives_by_central_differences(oracle, case, norm):
    B, heads, H, W, d, ks, extra = case
    q, k, v, w, bias, g = draw(82, *case)
    grads = oracle.backward_explicit(q, k, v, w, g, H, W, norm=norm, extra=extra)
    r = np.random.default_rng(5)
    loss = lambda q_, k_, v_, w_, b_: float(
        (oracle.forward_explicit(q_, k_, v_, w_, b_, H, W, norm=norm, extra=extra) * g).sum())
    x = (q, k, v, w, bias)
    for trial in range(4):
        dirs = [r.normal(size=a.shape) * (trial == 3 or i == trial % 3 or (i > 2 and trial == 2))
                for i, a in enumerate(x)]
        h = 1e-6
        plus = loss(*(a + h * d_ for a, d_ in zip(x, dirs)))
        minus = loss(*(a - h * d_ for a, d_ in zip(x, dirs)))
        want = (plus - minus) / (2 * h)
        got = sum(float((gr * d_).sum()) for gr, d_ in zip(grads, dirs))
        assert abs(got - want) <= 1e-6 * max(1.0, abs(want)), (trial, got, want)


def test_structure_of_the_gradients(oracle):
    B, heads, H, W, d, ks, extra = 1, 2, 5, 4, 6, 3, 0
    q, k, v, w, bias, g = draw(83, B, heads, H, W, d, ks)
    dq, dk, dv, dw, dbias = oracle.backward_explicit(q, k, v, w, g, H, W)
    # scaling q or k leaves the output unchanged: the gradients are orthogonal to the rows
    assert np.abs((dq * q).sum(-1)).max() < 1e-12
    assert np.abs((dk * k).sum(-1)).max() < 1e-12
    # the bias reaches every grid token once
    np.testing.assert_allclose(dbias, g.sum(axis=(0, 2)), atol=1e-12)
    # with all values equal the normalised attention returns that value whatever q and k are
    v0 = np.broadcast_to(np.random.default_rng(1).normal(size=(1, heads, 1, d)), v.shape).copy()
    dq0, dk0, _, _, _ = oracle.backward_explicit(q, k, v0, w, g, H, W, branches=oracle.BRANCH_LINEAR)
    assert np.abs(dq0).max() < 1e-12 and np.abs(dk0).max() < 1e-12
    # the rows of the normalised similarity sum to one: so do the weights g_t spreads over dv
    _, _, dv1, _, _ = oracle.backward_explicit(q, k, v, w, g, H, W, branches=oracle.BRANCH_LINEAR)
    np.testing.assert_allclose(dv1.sum(axis=2), g.sum(axis=2), atol=1e-12)
    # the residual connection passes g straight to dq
    dq2 = oracle.backward_explicit(q, k, v, w, g, H, W, residual=True)[0]
    np.testing.assert_allclose(dq2 - dq, g, atol=1e-13)


def test_reassociated_backward_at_a_larger_size(oracle):
    case = (1, 2, 12, 14, 16, 5, 1)
    B, heads, H, W, d, ks, extra = case
    q, k, v, w, bias, g = draw(84, *case)
    for norm in (0, 1):
        a = oracle.backward_explicit(q, k, v, w, g, H, W, norm=norm, extra=extra)
        f = oracle.backward(q, k, v, w, g, H, W, norm=norm, extra=extra)
        for x, y in zip(a, f):
            np.testing.assert_allclose(y, x, rtol=1e-9, atol=1e-10)
    assert oracle.backward(q, k, v, w, g, H, W, extra=extra, with_bias=False)[4] is None


POOLED = [(2, 2, 6, 8, 4, 3, 2), (1, 3, 7, 5, 3, 5, 2), (1, 1, 9, 9, 2, 3, 3), (1, 2, 1, 6, 4, 3, 2)]


@pytest.mark.parametrize("case", POOLED)
@pytest.mark.parametrize("norm", [0, 1])
@pytest.mark.parametrize("branches", [3, 1, 2])
def test_pooled_gradients_equal_autograd_of_the_definition(oracle, case, norm, branches):
    """Downsampling layer: pooled queries against all keys, DWConv of stride `pool`, residual
    query -- in plain torch ops (matmul, conv2d with a stride), differentiated by autograd."""
    B, heads, H, W, d, ks, pool = case
    r = np.random.default_rng(85)
    hq, wq = -(-H // pool), -(-W // pool)
    q, g = r.normal(size=(B, heads, hq * wq, d)), r.normal(size=(B, heads, hq * wq, d))
    k, v = r.normal(size=(B, heads, H * W, d)), r.normal(size=(B, heads, H * W, d))
    w, bias = r.normal(size=(heads, d, ks, ks)) * 0.3, r.normal(size=(heads, d))
    eps = 0.9 * math.sqrt(d)
    residual = bool(branches & 1)
    tq, tk, tv, tw, tb = (torch.tensor(a, requires_grad=True) for a in (q, k, v, w, bias))
    out = torch.zeros_like(tq)
    if branches & 1:
        qh = tq / torch.clamp(tq.norm(dim=-1, keepdim=True), min=eps)
        kh = tk / torch.clamp(tk.norm(dim=-1, keepdim=True), min=eps)
        A = 0.5 + qh @ kh.transpose(-1, -2) / PI
        lin = A @ tv
        out = out + (lin / A.sum(-1, keepdim=True) if norm == 0 else lin)
    if branches & 2:
        x = tv.reshape(B, heads, H, W, d).permute(0, 1, 4, 2, 3).reshape(B, heads * d, H, W)
        y = torch.nn.functional.conv2d(x, tw.reshape(heads * d, 1, ks, ks), tb.reshape(-1), stride=pool,
                                       padding=ks // 2, groups=heads * d)
        out = out + y.reshape(B, heads, d, hq, wq).permute(0, 1, 3, 4, 2).reshape(B, heads, hq * wq, d)
    if residual:
        out = out + tq
    np.testing.assert_allclose(
        out.detach().numpy(),
        oracle.forward_pooled_explicit(q, k, v, w, bias, H, W, pool=pool, residual=residual, norm=norm,
                                       branches=branches, eps=eps), atol=1e-12)
    (out * torch.tensor(g)).sum().backward()
    want = [t.grad.numpy() if t.grad is not None else np.zeros(t.shape) for t in (tq, tk, tv, tw, tb)]
    got = oracle.backward_pooled_explicit(q, k, v, w, g, H, W, pool=pool, residual=residual, norm=norm,
                                          branches=branches, eps=eps)
    for name, a, b in zip(("dq", "dk", "dv", "dw", "dbias"), got, want):
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-10, err_msg=name)


def test_pooled_backward_with_stride_one_is_the_ordinary_backward(oracle):
    B, heads, H, W, d, ks, extra = CASES[0]
    q, k, v, w, bias, g = draw(86, *CASES[0])
    a = oracle.backward_explicit(q, k, v, w, g, H, W, residual=True)
    b = oracle.backward_pooled_explicit(q, k, v, w, g, H, W, pool=1, residual=True)
    for x, y in zip(a, b):
        np.testing.assert_allclose(y, x, atol=1e-12)
