"""ctypes front end of oracle/castling_oracle.c (test infrastructure only).

All arrays are float64 numpy arrays, C-contiguous:
  q, k, v, out : [B, heads, N, d]  (N = grid_h * grid_w, token n = y*grid_w + x)
  w            : [heads, d, ks, ks]
  bias         : [heads, d] or None
See the C file's header for which passage of the paper each function follows.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

BRANCH_LINEAR = 1
BRANCH_DWCONV = 2
BRANCH_ALL = 3
NORM_ROWSUM = 0
NORM_NONE = 1
DEFAULT_EPS = 1e-12

_lib = None
_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int64)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.oracle_l2_normalize.argtypes = [_dp, C.c_int64, C.c_int, C.c_double, _dp]
        L.oracle_sim_angular.argtypes = [_dp, _dp, C.c_int, C.c_int, C.c_double, _dp]
        L.oracle_sim_linear.argtypes = [_dp, _dp, C.c_int, C.c_int, C.c_double, _dp]
        L.oracle_series_coeff.argtypes = [C.c_int]
        L.oracle_series_coeff.restype = C.c_double
        L.oracle_sim_series.argtypes = [C.c_double, C.c_int]
        L.oracle_sim_series.restype = C.c_double
        L.oracle_dwconv.argtypes = [_dp, _dp, _dp] + [C.c_int] * 6 + [_dp]
        fwd = [_dp] * 5 + [C.c_int] * 6 + [C.c_int, C.c_uint, C.c_double, C.c_int]
        L.oracle_forward_explicit.argtypes = fwd + [_dp]
        L.oracle_forward.argtypes = fwd + [_dp]
        L.oracle_forward_explicit_rows.argtypes = fwd + [_ip, _ip, C.c_int64, _dp]
        pooled = [_dp] * 5 + [C.c_int] * 9 + [C.c_uint, C.c_double, _dp]
        L.oracle_forward_pooled_explicit.argtypes = pooled
        L.oracle_forward_pooled.argtypes = pooled
        bwd = [_dp] * 5 + [C.c_int] * 7 + [C.c_uint, C.c_double, C.c_int, C.c_int] + [_dp] * 5
        L.oracle_backward_explicit.argtypes = bwd
        L.oracle_backward.argtypes = bwd
        L.oracle_backward_explicit_rows.argtypes = \
            [_dp] * 5 + [C.c_int] * 7 + [C.c_uint, C.c_double, C.c_int, C.c_int] + \
            [_ip, _ip, C.c_int64] + [_dp] * 3
        L.oracle_backward_explicit_rows.restype = None
        L.oracle_backward_pooled_explicit.argtypes = \
            [_dp] * 5 + [C.c_int] * 9 + [C.c_uint, C.c_double] + [_dp] * 5
        L.oracle_state.argtypes = [_dp, _dp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, _dp]
        L.oracle_softmax_probs.argtypes = [_dp, _dp, C.c_int, C.c_int, C.c_int, C.c_double,
                                           C.c_double, _dp]
        L.oracle_sparse_attn.argtypes = [_dp, _dp, _dp] + [C.c_int] * 5 + [C.c_double] * 3 + \
            [_dp, C.POINTER(C.c_int64)]
        L.oracle_angular_attn.argtypes = [_dp, _dp, _dp] + [C.c_int] * 5 + [C.c_double, _dp]
        for name in ("oracle_softmax_probs", "oracle_sparse_attn", "oracle_angular_attn"):
            getattr(L, name).restype = None
        L.oracle_num_threads.restype = C.c_int
        L.oracle_set_num_threads.argtypes = [C.c_int]
        for name in ("oracle_l2_normalize", "oracle_sim_angular", "oracle_sim_linear",
                     "oracle_dwconv", "oracle_forward_explicit", "oracle_forward",
                     "oracle_forward_explicit_rows", "oracle_state", "oracle_set_num_threads"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(_dp)


def l2_normalize(x, eps=DEFAULT_EPS):
    x = _f64(x)
    out = np.empty_like(x)
    d = x.shape[-1]
    lib().oracle_l2_normalize(_p(x), x.size // d, d, eps, _p(out))
    return out


def sim_angular(q, k, eps=DEFAULT_EPS):
    """Eq. 5 similarity matrix of one head: q, k are [N, d] -> [N, N]."""
    q, k = _f64(q), _f64(k)
    N, d = q.shape
    A = np.empty((N, N), dtype=np.float64)
    lib().oracle_sim_angular(_p(q), _p(k), N, d, eps, _p(A))
    return A


def sim_linear(q, k, eps=DEFAULT_EPS):
    """Linear-angular terms of Eq. 8 for one head: [N, d], [N, d] -> [N, N]."""
    q, k = _f64(q), _f64(k)
    N, d = q.shape
    A = np.empty((N, N), dtype=np.float64)
    lib().oracle_sim_linear(_p(q), _p(k), N, d, eps, _p(A))
    return A


def series_coeff(k: int) -> float:
    return lib().oracle_series_coeff(int(k))


def sim_series(x: float, order: int) -> float:
    return lib().oracle_sim_series(float(x), int(order))


def dwconv(v, w, bias, grid_h, grid_w):
    v, w = _f64(v), _f64(w)
    bias = None if bias is None else _f64(bias)
    B, heads, N, d = v.shape
    assert N == grid_h * grid_w and w.shape[:2] == (heads, d) and w.shape[2] == w.shape[3]
    out = np.empty_like(v)
    lib().oracle_dwconv(_p(v), _p(w), _p(bias), B, heads, grid_h, grid_w, d, w.shape[2], _p(out))
    return out


def _fwd_args(q, k, v, w, bias, grid_h, grid_w, norm, branches, eps, extra=0):
    q, k, v, w = _f64(q), _f64(k), _f64(v), _f64(w)
    bias = None if bias is None else _f64(bias)
    B, heads, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    assert N == extra + grid_h * grid_w and w.shape[:2] == (heads, d) and w.shape[2] == w.shape[3]
    keep = (q, k, v, w, bias)
    args = [_p(q), _p(k), _p(v), _p(w), _p(bias), B, heads, grid_h, grid_w, d, w.shape[2],
            int(norm), int(branches), float(eps), int(extra)]
    return keep, args, q.shape


def forward_explicit(q, k, v, w, bias, grid_h, grid_w, norm=NORM_ROWSUM, branches=BRANCH_ALL,
                     eps=DEFAULT_EPS, extra=0):
    """The layer by its definition (explicit N x N similarity); small N only.  `extra` tokens in
    front of each unit's grid tokens are not on the grid (class tokens)."""
    keep, args, shape = _fwd_args(q, k, v, w, bias, grid_h, grid_w, norm, branches, eps, extra)
    out = np.empty(shape, dtype=np.float64)
    lib().oracle_forward_explicit(*args, _p(out))
    return out


def forward(q, k, v, w, bias, grid_h, grid_w, norm=NORM_ROWSUM, branches=BRANCH_ALL,
            eps=DEFAULT_EPS, extra=0):
    """The layer by the reassociated (K^T V state) form; any N."""
    keep, args, shape = _fwd_args(q, k, v, w, bias, grid_h, grid_w, norm, branches, eps, extra)
    out = np.empty(shape, dtype=np.float64)
    lib().oracle_forward(*args, _p(out))
    return out


def forward_explicit_rows(q, k, v, w, bias, grid_h, grid_w, units, tokens, norm=NORM_ROWSUM,
                          branches=BRANCH_ALL, eps=DEFAULT_EPS, extra=0):
    """Definition on selected rows (unit = b*heads + h, token); returns [nrows, d]."""
    keep, args, shape = _fwd_args(q, k, v, w, bias, grid_h, grid_w, norm, branches, eps, extra)
    units = np.ascontiguousarray(units, dtype=np.int64)
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    order = np.argsort(units, kind="stable")      # group rows of one unit together
    us, ts = np.ascontiguousarray(units[order]), np.ascontiguousarray(tokens[order])
    out_sorted = np.empty((len(us), shape[-1]), dtype=np.float64)
    lib().oracle_forward_explicit_rows(*args, us.ctypes.data_as(_ip), ts.ctypes.data_as(_ip),
                                       len(us), _p(out_sorted))
    out = np.empty_like(out_sorted)
    out[order] = out_sorted
    return out


def _pooled(fn, q, k, v, w, bias, grid_h, grid_w, pool, residual, norm, branches, eps):
    q, k, v, w = _f64(q), _f64(k), _f64(v), _f64(w)
    bias = None if bias is None else _f64(bias)
    B, heads, N, d = k.shape
    nq = -(-grid_h // pool) * -(-grid_w // pool)
    assert v.shape == k.shape and N == grid_h * grid_w and q.shape == (B, heads, nq, d)
    assert w.shape[:2] == (heads, d) and w.shape[2] == w.shape[3]
    out = np.empty(q.shape, dtype=np.float64)
    fn(_p(q), _p(k), _p(v), _p(w), _p(bias), B, heads, grid_h, grid_w, d, w.shape[2], int(pool),
       int(bool(residual)), int(norm), int(branches), float(eps), _p(out))
    return out


def forward_pooled_explicit(q, k, v, w, bias, grid_h, grid_w, pool=2, residual=True,
                            norm=NORM_ROWSUM, branches=BRANCH_ALL, eps=DEFAULT_EPS):
    """Downsampling layer by its definition: pooled queries on every pool-th row and column of
    the grid of K and V, DWConv rows of those positions, optional residual query; small N."""
    return _pooled(lib().oracle_forward_pooled_explicit, q, k, v, w, bias, grid_h, grid_w, pool,
                   residual, norm, branches, eps)


def forward_pooled(q, k, v, w, bias, grid_h, grid_w, pool=2, residual=True, norm=NORM_ROWSUM,
                   branches=BRANCH_ALL, eps=DEFAULT_EPS):
    """The same by the reassociated form; any N."""
    return _pooled(lib().oracle_forward_pooled, q, k, v, w, bias, grid_h, grid_w, pool, residual,
                   norm, branches, eps)


def _backward(fn, q, k, v, w, g, grid_h, grid_w, norm, branches, eps, extra, residual, with_bias):
    q, k, v, w, g = _f64(q), _f64(k), _f64(v), _f64(w), _f64(g)
    B, heads, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and g.shape == q.shape
    assert N == extra + grid_h * grid_w and w.shape[:2] == (heads, d) and w.shape[2] == w.shape[3]
    dq, dk, dv = (np.empty(q.shape, dtype=np.float64) for _ in range(3))
    dw = np.empty(w.shape, dtype=np.float64)
    dbias = np.empty((heads, d), dtype=np.float64) if with_bias else None
    fn(_p(q), _p(k), _p(v), _p(w), _p(g), B, heads, grid_h, grid_w, d, w.shape[2], int(norm),
       int(branches), float(eps), int(extra), int(bool(residual)), _p(dq), _p(dk), _p(dv), _p(dw),
       _p(dbias))
    return dq, dk, dv, dw, dbias


def backward_explicit(q, k, v, w, g, grid_h, grid_w, norm=NORM_ROWSUM, branches=BRANCH_ALL,
                      eps=DEFAULT_EPS, extra=0, residual=False, with_bias=True):
    """Gradients (dq, dk, dv, dw, dbias) of the layer given g = dLoss/dout, by differentiating
    the definition (explicit N x N similarity); small N only."""
    return _backward(lib().oracle_backward_explicit, q, k, v, w, g, grid_h, grid_w, norm, branches,
                     eps, extra, residual, with_bias)


def backward(q, k, v, w, g, grid_h, grid_w, norm=NORM_ROWSUM, branches=BRANCH_ALL,
             eps=DEFAULT_EPS, extra=0, residual=False, with_bias=True):
    """The same through the reassociated state; any N."""
    return _backward(lib().oracle_backward, q, k, v, w, g, grid_h, grid_w, norm, branches, eps,
                     extra, residual, with_bias)


def backward_explicit_rows(q, k, v, w, g, grid_h, grid_w, units, tokens, norm=NORM_ROWSUM,
                           branches=BRANCH_ALL, eps=DEFAULT_EPS, extra=0, residual=False):
    """Gradient rows (dq, dk, dv), each [nrows, d], with respect to the selected tokens
    (unit = b*heads + h, token), by differentiating the definition; any N, O(N^2 d) per unit
    that has a selected row.  Uses nothing of the reassociated form."""
    q, k, v, w, g = _f64(q), _f64(k), _f64(v), _f64(w), _f64(g)
    B, heads, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and g.shape == q.shape
    assert N == extra + grid_h * grid_w and w.shape[:2] == (heads, d) and w.shape[2] == w.shape[3]
    units = np.ascontiguousarray(units, dtype=np.int64)
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    assert units.shape == tokens.shape and units.ndim == 1
    assert units.min() >= 0 and units.max() < B * heads and tokens.min() >= 0 and tokens.max() < N
    order = np.argsort(units, kind="stable")      # rows of one unit next to each other
    us, ts = np.ascontiguousarray(units[order]), np.ascontiguousarray(tokens[order])
    rows = [np.empty((len(us), d), dtype=np.float64) for _ in range(3)]
    lib().oracle_backward_explicit_rows(
        _p(q), _p(k), _p(v), _p(w), _p(g), B, heads, grid_h, grid_w, d, w.shape[2], int(norm),
        int(branches), float(eps), int(extra), int(bool(residual)), us.ctypes.data_as(_ip),
        ts.ctypes.data_as(_ip), len(us), _p(rows[0]), _p(rows[1]), _p(rows[2]))
    out = []
    for r in rows:
        o = np.empty_like(r)
        o[order] = r
        out.append(o)
    return tuple(out)


def backward_pooled_explicit(q, k, v, w, g, grid_h, grid_w, pool=2, residual=True, norm=NORM_ROWSUM,
                             branches=BRANCH_ALL, eps=DEFAULT_EPS, with_bias=True):
    """Gradients (dq, dk, dv, dw, dbias) of the downsampling layer (forward_pooled_explicit) given
    g = dLoss/dout [B, heads, Nq, d], by differentiating its definition; small N only."""
    q, k, v, w, g = _f64(q), _f64(k), _f64(v), _f64(w), _f64(g)
    B, heads, N, d = k.shape
    nq = -(-grid_h // pool) * -(-grid_w // pool)
    assert v.shape == k.shape and N == grid_h * grid_w and q.shape == (B, heads, nq, d)
    assert g.shape == q.shape and w.shape[:2] == (heads, d) and w.shape[2] == w.shape[3]
    dq = np.empty(q.shape, dtype=np.float64)
    dk, dv = np.empty(k.shape, dtype=np.float64), np.empty(k.shape, dtype=np.float64)
    dw = np.empty(w.shape, dtype=np.float64)
    dbias = np.empty((heads, d), dtype=np.float64) if with_bias else None
    lib().oracle_backward_pooled_explicit(
        _p(q), _p(k), _p(v), _p(w), _p(g), B, heads, grid_h, grid_w, d, w.shape[2], int(pool),
        int(bool(residual)), int(norm), int(branches), float(eps), _p(dq), _p(dk), _p(dv), _p(dw),
        _p(dbias))
    return dq, dk, dv, dw, dbias


def state(k, v, eps=DEFAULT_EPS):
    """[B, heads, d+1, d+1] = [K_hat | 1]^T [V | 1] per unit."""
    k, v = _f64(k), _f64(v)
    B, heads, N, d = k.shape
    st = np.empty((B, heads, d + 1, d + 1), dtype=np.float64)
    lib().oracle_state(_p(k), _p(v), B, heads, N, d, eps, _p(st))
    return st


def softmax_probs(q, k, normalize=True, scale=1.0, eps=DEFAULT_EPS):
    """One head: q, k [N, d] -> P [N, N], the softmax attention map inside Eq. 10."""
    q, k = _f64(q), _f64(k)
    N, d = q.shape
    P = np.empty((N, N), dtype=np.float64)
    lib().oracle_softmax_probs(_p(q), _p(k), N, d, int(bool(normalize)), scale, eps, _p(P))
    return P


def sparse_attn(q, k, v, thr, normalize=True, scale=1.0, eps=DEFAULT_EPS):
    """Eq. 10 applied to V: (out [B, heads, N, d], kept entries per unit [B, heads])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, heads, N, d = q.shape
    out = np.empty_like(q)
    nnz = np.zeros((B, heads), dtype=np.int64)
    lib().oracle_sparse_attn(_p(q), _p(k), _p(v), B, heads, N, d, int(bool(normalize)), scale,
                             thr, eps, _p(out), nnz.ctypes.data_as(C.POINTER(C.c_int64)))
    return out, nnz


def angular_attn(q, k, v, norm=NORM_ROWSUM, eps=DEFAULT_EPS):
    """Attention with the exact angular kernel of Eq. 5 instead of its linear terms."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, heads, N, d = q.shape
    out = np.empty_like(q)
    lib().oracle_angular_attn(_p(q), _p(k), _p(v), B, heads, N, d, norm, eps, _p(out))
    return out


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(int(n))
