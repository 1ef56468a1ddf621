"""Property-based checks of the oracle over random small shapes (hypothesis): facts that hold
for every input of the layer as Eq. 3, 8, 9 define it, so that a mistake in an index, a
stride or a special case of the oracle shows on some drawn shape.  CPU only."""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings
from hypothesis import strategies as st

SETTINGS = dict(max_examples=60, deadline=None, derandomize=True,
                suppress_health_check=[HealthCheck.function_scoped_fixture, HealthCheck.too_slow])


@st.composite
def layer_case(draw, max_side=9):
    B = draw(st.integers(1, 2))
    heads = draw(st.integers(1, 3))
    H = draw(st.integers(1, max_side))
    W = draw(st.integers(1, max_side))
    d = draw(st.integers(1, 12))
    ks = draw(st.sampled_from([1, 3, 5, 7, 9]))
    extra = draw(st.integers(0, 3))
    norm = draw(st.sampled_from([0, 1]))
    branches = draw(st.sampled_from([1, 2, 3]))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    r = np.random.default_rng(seed)
    N = extra + H * W
    q, k, v = (r.normal(size=(B, heads, N, d)) for _ in range(3))
    # some rows under the floor of the norm, some exactly zero
    eps = draw(st.sampled_from([1e-12, 0.8 * np.sqrt(d)]))
    if draw(st.booleans()):
        q[0, 0, r.integers(N)] = 0.0
        k[0, 0, r.integers(N)] = 0.0
    w = r.normal(size=(heads, d, ks, ks)) * 0.3
    bias = r.normal(size=(heads, d)) if draw(st.booleans()) else None
    return dict(q=q, k=k, v=v, w=w, bias=bias, H=H, W=W, extra=extra, norm=norm, branches=branches,
                eps=eps, rng=r)


def _fwd(oracle, c, fn=None, **over):
    a = {**c, **over}
    return (fn or oracle.forward)(a["q"], a["k"], a["v"], a["w"], a["bias"], a["H"], a["W"], norm=a["norm"],
                                  branches=a["branches"], eps=a["eps"], extra=a["extra"])


@settings(**SETTINGS)
@given(c=layer_case())
def test_reassociated_form_equals_the_definition(oracle, c):
    """Sec. 3.1: (Q_hat K_hat^T) V regrouped as Q_hat (K_hat^T V) is the same numbers."""
    want = _fwd(oracle, c, fn=oracle.forward_explicit)
    got = _fwd(oracle, c)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-11)
    B, heads, N, d = c["q"].shape
    r = c["rng"]
    units, tokens = r.integers(B * heads, size=5), r.integers(N, size=5)
    rows = oracle.forward_explicit_rows(c["q"], c["k"], c["v"], c["w"], c["bias"], c["H"], c["W"], units,
                                        tokens, norm=c["norm"], branches=c["branches"], eps=c["eps"],
                                        extra=c["extra"])
    np.testing.assert_allclose(rows, want.reshape(B * heads, N, d)[units, tokens], rtol=1e-12, atol=1e-13)


@settings(**SETTINGS)
@given(c=layer_case())
def test_linear_in_v_and_in_the_filters(oracle, c):
    """Eq. 9 is linear in V for fixed Q, K (both branches), and the DWConv term in its filters."""
    c = dict(c, bias=None)
    v2 = c["rng"].normal(size=c["v"].shape)
    both = _fwd(oracle, c, v=2.0 * c["v"] - 3.0 * v2)
    np.testing.assert_allclose(both, 2.0 * _fwd(oracle, c) - 3.0 * _fwd(oracle, c, v=v2), rtol=1e-9,
                               atol=1e-10)
    if c["branches"] == 2:
        w2 = c["rng"].normal(size=c["w"].shape)
        np.testing.assert_allclose(_fwd(oracle, c, w=c["w"] + w2),
                                   _fwd(oracle, c) + _fwd(oracle, c, w=w2), rtol=1e-9, atol=1e-10)


@settings(**SETTINGS)
@given(c=layer_case())
def test_weights_are_a_convex_combination(oracle, c):
    """Eq. 3 with the similarity of Eq. 8 (every A_tj in [1/2 - 1/pi, 1/2 + 1/pi] > 0): each
    normalised output row lies between the channel-wise minimum and maximum of V, and is the
    constant when V is constant over the tokens."""
    c = dict(c, branches=1, norm=0)
    out = _fwd(oracle, c)
    lo = c["v"].min(axis=2, keepdims=True)
    hi = c["v"].max(axis=2, keepdims=True)
    assert np.all(out >= lo - 1e-12) and np.all(out <= hi + 1e-12)
    const = np.broadcast_to(c["v"][:, :, :1], c["v"].shape).copy()
    np.testing.assert_allclose(_fwd(oracle, c, v=const), const, rtol=1e-12, atol=1e-13)


@settings(**SETTINGS)
@given(c=layer_case())
def test_row_scaling_and_token_order(oracle, c):
    """The unit rows of Eq. 3 / Eq. 8: positive scaling of a query or key row above the norm
    floor changes nothing; the sums over j do not depend on the order of the keys, and a
    permutation of the queries permutes the output rows."""
    c = dict(c, branches=1, eps=1e-12)
    r = c["rng"]
    B, heads, N, d = c["q"].shape
    base = _fwd(oracle, c)
    sq = r.uniform(0.1, 10.0, size=(B, heads, N, 1))
    sk = r.uniform(0.1, 10.0, size=(B, heads, N, 1))
    np.testing.assert_allclose(_fwd(oracle, c, q=c["q"] * sq, k=c["k"] * sk), base, rtol=1e-9, atol=1e-10)
    pk, pq = r.permutation(N), r.permutation(N)
    np.testing.assert_allclose(_fwd(oracle, c, k=c["k"][:, :, pk], v=c["v"][:, :, pk]), base, rtol=1e-9,
                               atol=1e-10)
    np.testing.assert_allclose(_fwd(oracle, c, q=c["q"][:, :, pq]), base[:, :, pq], rtol=1e-12, atol=1e-13)


@settings(**SETTINGS)
@given(c=layer_case(max_side=7))
def test_gradients_are_the_derivative_of_the_forward(oracle, c):
    """<g, f(x + h e) - f(x - h e)> / 2h = <grad, e> along a random direction in (q, k, v, w),
    for the reassociated backward and for the sampled rows of the definition's gradient."""
    if c["bias"] is None:
        c = dict(c, bias=np.zeros(c["w"].shape[:2]))
    r = c["rng"]
    c = dict(c, eps=1e-12)           # keep away from the kink of max(|x|, eps)
    c["q"] = c["q"] + 0.5 * np.sign(c["q"] + 1e-300)
    c["k"] = c["k"] + 0.5 * np.sign(c["k"] + 1e-300)
    g = r.normal(size=c["q"].shape)
    dirs = {n: r.normal(size=c[n].shape) for n in ("q", "k", "v", "w")}
    h = 1e-5
    plus = _fwd(oracle, c, **{n: c[n] + h * dirs[n] for n in dirs})
    minus = _fwd(oracle, c, **{n: c[n] - h * dirs[n] for n in dirs})
    numeric = np.sum(g * (plus - minus)) / (2 * h)
    grads = oracle.backward(c["q"], c["k"], c["v"], c["w"], g, c["H"], c["W"], norm=c["norm"],
                            branches=c["branches"], eps=c["eps"], extra=c["extra"])
    analytic = sum(np.sum(grads[i] * dirs[n]) for i, n in enumerate(("q", "k", "v", "w")))
    scale = sum(np.linalg.norm(grads[i]) * np.linalg.norm(dirs[n]) for i, n in enumerate(("q", "k", "v", "w")))
    assert abs(numeric - analytic) <= 1e-6 * max(scale, 1e-6)
    B, heads, N, d = c["q"].shape
    units, tokens = r.integers(B * heads, size=4), r.integers(N, size=4)
    rows = oracle.backward_explicit_rows(c["q"], c["k"], c["v"], c["w"], g, c["H"], c["W"], units, tokens,
                                         norm=c["norm"], branches=c["branches"], eps=c["eps"],
                                         extra=c["extra"])
    for a, full in zip(rows, grads[:3]):
        np.testing.assert_allclose(a, full.reshape(B * heads, N, d)[units, tokens], rtol=1e-8, atol=1e-10)
