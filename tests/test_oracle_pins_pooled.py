"""Pins of the oracle's downsampling-layer functions (pooled queries, residual query; Sec. 3.1
and the last row of Table 1) against things other than themselves: torch's strided grouped
conv2d, numpy matmul on the explicit similarity matrix, and the already pinned unpooled layer
evaluated with the pooled queries placed on the positions they stand at."""
import math

import numpy as np
import pytest
import torch

PI = math.pi


def draw(seed, B, heads, H, W, d, ks, pool):
    r = np.random.default_rng(seed)
    nq = -(-H // pool) * -(-W // pool)
    q = r.normal(size=(B, heads, nq, d))
    k = r.normal(size=(B, heads, H * W, d))
    v = r.normal(size=(B, heads, H * W, d))
    w = r.normal(size=(heads, d, ks, ks)) * 0.3
    bias = r.normal(size=(heads, d))
    return q, k, v, w, bias


SHAPES = [(2, 2, 6, 8, 4, 3, 2), (1, 3, 7, 5, 3, 5, 2), (1, 1, 9, 9, 2, 3, 3), (1, 2, 1, 6, 4, 3, 2),
          (2, 1, 5, 1, 3, 1, 2)]


@pytest.mark.parametrize("shape", SHAPES)
def test_convolution_rows_are_a_strided_conv2d(oracle, shape):
    B, heads, H, W, d, ks, pool = shape
    q, k, v, w, bias = draw(61, *shape)
    got = oracle.forward_pooled_explicit(q, k, v, w, bias, H, W, pool=pool, residual=False,
                                         branches=oracle.BRANCH_DWCONV)
    x = torch.from_numpy(v).reshape(B, heads, H, W, d).permute(0, 1, 4, 2, 3).reshape(B, heads * d, H, W)
    y = torch.nn.functional.conv2d(x, torch.from_numpy(w).reshape(heads * d, 1, ks, ks),
                                   torch.from_numpy(bias).reshape(-1), stride=pool, padding=ks // 2,
                                   groups=heads * d)
    hq, wq = -(-H // pool), -(-W // pool)
    assert y.shape[-2:] == (hq, wq)
    want = y.reshape(B, heads, d, hq, wq).permute(0, 1, 3, 4, 2).reshape(B, heads, hq * wq, d).numpy()
    np.testing.assert_allclose(got, want, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("norm", [0, 1])
def test_linear_rows_by_matmul(oracle, shape, norm):
    B, heads, H, W, d, ks, pool = shape
    q, k, v, w, bias = draw(62, *shape)
    got = oracle.forward_pooled_explicit(q, k, v, w, bias, H, W, pool=pool, residual=False,
                                         norm=norm, branches=oracle.BRANCH_LINEAR)
    qh = q / np.linalg.norm(q, axis=-1, keepdims=True)
    kh = k / np.linalg.norm(k, axis=-1, keepdims=True)
    A = 0.5 + np.einsum("bhtc,bhjc->bhtj", qh, kh) / PI          # Nq x N similarity, Eq. 8
    want = A @ v
    if norm == 0:
        want = want / A.sum(-1, keepdims=True)
    np.testing.assert_allclose(got, want, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("norm", [0, 1])
def test_pooled_layer_is_the_layer_at_the_query_positions(oracle, shape, norm):
    """Put the pooled queries on the positions they stand at, anything in between: the full
    layer's rows at those positions are the downsampling layer's rows."""
    B, heads, H, W, d, ks, pool = shape
    q, k, v, w, bias = draw(63, *shape)
    hq, wq = -(-H // pool), -(-W // pool)
    q_full = np.random.default_rng(7).normal(size=(B, heads, H, W, d))
    q_full[:, :, ::pool, ::pool] = q.reshape(B, heads, hq, wq, d)
    full = oracle.forward_explicit(q_full.reshape(B, heads, H * W, d), k, v, w, bias, H, W, norm=norm)
    want = full.reshape(B, heads, H, W, d)[:, :, ::pool, ::pool].reshape(B, heads, hq * wq, d)
    got = oracle.forward_pooled_explicit(q, k, v, w, bias, H, W, pool=pool, residual=False, norm=norm)
    np.testing.assert_allclose(got, want, atol=1e-12)
    # the residual connection adds the pooled query itself
    res = oracle.forward_pooled_explicit(q, k, v, w, bias, H, W, pool=pool, residual=True, norm=norm)
    np.testing.assert_allclose(res - got, q, atol=1e-12)
    # with a stride of one the two layers are the same thing
    one = oracle.forward_pooled_explicit(q_full.reshape(B, heads, H * W, d), k, v, w, bias, H, W,
                                         pool=1, residual=False, norm=norm)
    np.testing.assert_allclose(one, full, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES + [(1, 2, 20, 24, 16, 7, 2)])
@pytest.mark.parametrize("norm", [0, 1])
def test_reassociated_form_equals_the_definition(oracle, shape, norm):
    B, heads, H, W, d, ks, pool = shape
    q, k, v, w, bias = draw(64, *shape)
    for branches in (oracle.BRANCH_ALL, oracle.BRANCH_LINEAR, oracle.BRANCH_DWCONV):
        for residual in (False, True):
            a = oracle.forward_pooled_explicit(q, k, v, w, bias, H, W, pool=pool, residual=residual,
                                               norm=norm, branches=branches)
            f = oracle.forward_pooled(q, k, v, w, bias, H, W, pool=pool, residual=residual,
                                      norm=norm, branches=branches)
            np.testing.assert_allclose(f, a, rtol=1e-10, atol=1e-10)


def test_constant_values_come_back(oracle):
    """With every v_j = c the normalised linear branch returns c for any query (rows of a
    stochastic matrix), so out = c + q with a zero filter."""
    B, heads, H, W, d, ks, pool = 1, 2, 6, 6, 4, 3, 2
    q, k, v, w, bias = draw(65, B, heads, H, W, d, ks, pool)
    c = np.random.default_rng(3).normal(size=(1, heads, 1, d))
    v = np.broadcast_to(c, v.shape).copy()
    out = oracle.forward_pooled(q, k, v, np.zeros_like(w), None, H, W, pool=pool, residual=True)
    np.testing.assert_allclose(out, c + q, atol=1e-12)
