"""Pins of the oracle's O(N^2) attention functions (CPU only): the masked softmax branch of
Eq. 10 and attention with the exact angular kernel of Eq. 4-5.  Each check ties the oracle to
something it does not compute itself: a closed form, a library routine, or an invariant."""
import numpy as np
import pytest
import scipy.special
import torch


def unit(x):
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def rand(seed, B=2, heads=2, N=24, d=8):
    r = np.random.default_rng(seed)
    return (r.normal(size=(B, heads, N, d)) for _ in range(3))


def test_softmax_probs_against_scipy(oracle):
    r = np.random.default_rng(1)
    q, k = r.normal(size=(17, 6)), r.normal(size=(17, 6))
    for normalize, scale in ((True, 1.0), (True, 4.0), (False, 6 ** -0.5)):
        a, b = (unit(q), unit(k)) if normalize else (q, k)
        want = scipy.special.softmax(scale * (a @ b.T), axis=1)
        got = oracle.softmax_probs(q, k, normalize=normalize, scale=scale)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-14)


def test_sparse_hand_example(oracle):
    # d = 1, N = 2: unit rows +1 / -1, logits [[1, -1], [-1, 1]], softmax rows
    # [e, 1/e] / (e + 1/e) = [0.880797078, 0.119202922]
    q = np.array([[[[2.0], [-3.0]]]])
    k = np.array([[[[0.5], [-4.0]]]])
    v = np.array([[[[10.0], [20.0]]]])
    hi, lo = np.e / (np.e + 1 / np.e), (1 / np.e) / (np.e + 1 / np.e)
    assert hi == pytest.approx(0.880797078, abs=1e-9)
    out, nnz = oracle.sparse_attn(q, k, v, thr=0.0)
    np.testing.assert_allclose(out.ravel(), [hi * 10 + lo * 20, lo * 10 + hi * 20], rtol=1e-14)
    assert nnz.item() == 4
    out, nnz = oracle.sparse_attn(q, k, v, thr=0.5)          # only the diagonal survives
    np.testing.assert_allclose(out.ravel(), [hi * 10, hi * 20], rtol=1e-14)
    assert nnz.item() == 2
    out, nnz = oracle.sparse_attn(q, k, v, thr=hi)           # strict comparison: nothing survives
    assert nnz.item() == 0 and not out.any()


def test_sparse_threshold_zero_is_softmax_attention(oracle):
    q, k, v = rand(2)
    out, nnz = oracle.sparse_attn(q, k, v, thr=0.0, normalize=True, scale=3.0)
    assert (nnz == q.shape[2] ** 2).all()
    tq, tk, tv = (torch.from_numpy(x) for x in (unit(q), unit(k), v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=3.0).numpy()
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-14)
    # raw rows with Eq. 1's 1/sqrt(d): torch's default scale
    out, _ = oracle.sparse_attn(q, k, v, thr=0.0, normalize=False, scale=q.shape[-1] ** -0.5)
    want = torch.nn.functional.scaled_dot_product_attention(
        *(torch.from_numpy(x) for x in (q, k, v))).numpy()
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-14)


def test_sparse_mask_properties(oracle):
    q, k, v = rand(3, B=1, heads=3, N=40, d=8)
    N = q.shape[2]
    prev = None
    for thr in (0.0, 0.01, 0.02, 0.05, 0.2, 1.0):
        out, nnz = oracle.sparse_attn(q, k, v, thr=thr, scale=5.0)
        # the same count and the same result from the probabilities, masked with numpy
        for h in range(3):
            P = oracle.softmax_probs(q[0, h], k[0, h], scale=5.0)
            M = np.where(P > thr, P, 0.0)
            assert nnz[0, h] == np.count_nonzero(M)
            np.testing.assert_allclose(out[0, h], M @ v[0, h], rtol=1e-13, atol=1e-15)
            assert (M.sum(axis=1) <= 1.0 + 1e-14).all()
        if prev is not None:
            assert (nnz <= prev).all()                       # a higher threshold keeps less
        prev = nnz
    assert (prev == 0).all()                                 # nothing exceeds 1


def test_sparse_identical_keys(oracle):
    # all keys equal: every probability is exactly 1/N, kept as a whole or not at all
    r = np.random.default_rng(4)
    N, d = 16, 4
    q, v = r.normal(size=(1, 1, N, d)), r.normal(size=(1, 1, N, d))
    k = np.tile(r.normal(size=(1, 1, 1, d)), (1, 1, N, 1))
    out, nnz = oracle.sparse_attn(q, k, v, thr=1.0 / N - 1e-9)
    assert nnz.item() == N * N
    np.testing.assert_allclose(out[0, 0], np.tile(v.mean(axis=2)[0, 0], (N, 1)), rtol=1e-13)
    out, nnz = oracle.sparse_attn(q, k, v, thr=1.0 / N + 1e-9)
    assert nnz.item() == 0 and not out.any()


def test_sparse_argmax_only(oracle):
    # a threshold just under each row's largest probability keeps exactly that entry
    q, k, v = rand(5, B=1, heads=1, N=12, d=6)
    P = oracle.softmax_probs(q[0, 0], k[0, 0], scale=8.0)
    thr = np.sort(P, axis=1)[:, -2].max()                    # above every runner-up
    if (P.max(axis=1) > thr).all():
        out, nnz = oracle.sparse_attn(q, k, v, thr=thr, scale=8.0)
        assert nnz.item() == 12
        j = P.argmax(axis=1)
        np.testing.assert_allclose(out[0, 0], P.max(axis=1)[:, None] * v[0, 0][j], rtol=1e-13)


def test_angular_attn_from_arccos(oracle):
    q, k, v = rand(6)
    for norm in (oracle.NORM_ROWSUM, oracle.NORM_NONE):
        got = oracle.angular_attn(q, k, v, norm=norm)
        A = 1.0 - np.arccos(np.clip(unit(q) @ np.swapaxes(unit(k), -1, -2), -1, 1)) / np.pi
        want = A @ v
        if norm == oracle.NORM_ROWSUM:
            want = want / A.sum(axis=-1, keepdims=True)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_angular_attn_orthonormal_closed_form(oracle):
    # q = k = an orthonormal basis: the kernel is 1 on the diagonal and 1/2 elsewhere
    N = d = 5
    r = np.random.default_rng(7)
    basis, _ = np.linalg.qr(r.normal(size=(d, d)))
    q = k = (basis * r.uniform(0.5, 3.0, size=(d, 1)))[None, None]   # rescaled rows, same directions
    v = r.normal(size=(1, 1, N, d))
    got = oracle.angular_attn(q, k, v)[0, 0]
    total = v[0, 0].sum(axis=0)
    want = (0.5 * total + 0.5 * v[0, 0]) / (1.0 + 0.5 * (N - 1))
    # arccos near 1 turns a rounding error delta of the dot product into sqrt(2 delta) ~ 1e-8
    np.testing.assert_allclose(got, want, rtol=1e-7, atol=1e-8)


def test_angular_attn_invariants(oracle):
    q, k, v = rand(8)
    base = oracle.angular_attn(q, k, v)
    r = np.random.default_rng(9)
    s = r.uniform(0.1, 10.0, size=q.shape[:3] + (1,))
    np.testing.assert_allclose(oracle.angular_attn(q * s, k / s, v), base, rtol=1e-10)
    perm = r.permutation(q.shape[2])
    np.testing.assert_allclose(oracle.angular_attn(q, k[:, :, perm], v[:, :, perm]), base, rtol=1e-11)
    const = np.ones_like(v) * 2.5
    np.testing.assert_allclose(oracle.angular_attn(q, k, const), const, rtol=1e-13)
    # convex combination of the values
    assert (base <= v.max(axis=2, keepdims=True) + 1e-12).all()
    assert (base >= v.min(axis=2, keepdims=True) - 1e-12).all()


def test_linear_terms_stay_within_the_truncation_gap(oracle):
    # Eq. 8: the linear terms differ from the exact kernel by the odd higher-order terms, whose
    # sum is at most 1/2 - 1/pi in magnitude (reached at x = +-1) and has the sign of x
    r = np.random.default_rng(10)
    q, k = r.normal(size=(30, 3)), r.normal(size=(30, 3))
    gap = oracle.sim_angular(q, k) - oracle.sim_linear(q, k)
    x = unit(q) @ unit(k).T
    assert np.abs(gap).max() <= 0.5 - 1 / np.pi + 1e-12
    assert (np.sign(gap[np.abs(x) > 1e-6]) == np.sign(x[np.abs(x) > 1e-6])).all()


def test_class_tokens_join_the_sums_but_not_the_convolution(oracle):
    """Tokens in front of the grid (class tokens): the linear branch treats all N = extra + H W
    tokens alike (it has no notion of position), the DWConv term exists on the grid only."""
    r = np.random.default_rng(11)
    B, heads, H, W, d, ks, E = 1, 2, 5, 6, 4, 3, 2
    N = E + H * W
    q, k, v = (r.normal(size=(B, heads, N, d)) for _ in range(3))
    w, bias = r.normal(size=(heads, d, ks, ks)), r.normal(size=(heads, d))
    for norm in (oracle.NORM_ROWSUM, oracle.NORM_NONE):
        full = oracle.forward_explicit(q, k, v, w, bias, H, W, norm=norm, extra=E)
        fast = oracle.forward(q, k, v, w, bias, H, W, norm=norm, extra=E)
        np.testing.assert_allclose(fast, full, rtol=1e-11, atol=1e-13)
        lin = oracle.forward_explicit(q, k, v, w, bias, H, W, norm=norm, extra=E,
                                      branches=oracle.BRANCH_LINEAR)
        # the linear branch is blind to the grid: the same N tokens as a 1 x N grid give it too
        flat = oracle.forward_explicit(q, k, v, np.zeros((heads, d, 1, 1)), None, 1, N, norm=norm,
                                       branches=oracle.BRANCH_LINEAR)
        np.testing.assert_allclose(lin, flat, rtol=1e-13, atol=1e-15)
        # class tokens get the linear branch only; grid tokens add the convolution of the grid part
        np.testing.assert_allclose(full[:, :, :E], lin[:, :, :E], rtol=1e-13)
        dw = oracle.dwconv(np.ascontiguousarray(v[:, :, E:]), w, bias, H, W)
        np.testing.assert_allclose(full[:, :, E:], lin[:, :, E:] + dw, rtol=1e-12, atol=1e-14)
        rows = oracle.forward_explicit_rows(q, k, v, w, bias, H, W, [0, 1, 1, 0], [0, 1, 7, N - 1],
                                            norm=norm, extra=E)
        np.testing.assert_allclose(rows, full.reshape(heads, N, d)[[0, 1, 1, 0], [0, 1, 7, N - 1]],
                                   rtol=1e-13)
    # extra = 0 is the layer as before
    np.testing.assert_array_equal(oracle.forward(q[:, :, E:], k[:, :, E:], v[:, :, E:], w, bias, H, W),
                                  oracle.forward(q[:, :, E:], k[:, :, E:], v[:, :, E:], w, bias, H, W, extra=0))
