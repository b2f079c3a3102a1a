"""Pins for the oracle's single layers: finite differences, adjoint identities,
special cases with known answers, BN identities, head closed forms.

The paper prints no worked numerical example, so the oracle is pinned to what
the mathematics fixes (Section 2, Eq. 3-5 define forward and chain rule).
"""
import numpy as np
import pytest

from oracle import ddg_oracle as orc

RNG = np.random.default_rng(1234)


def fd_grad(f, x, h=1e-5):
    """Central finite differences of scalar f at x (float64)."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = f(x)
        x[i] = old - h
        fm = f(x)
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


CONV_CASES = [(3, 1, 1), (3, 2, 1), (1, 1, 0), (1, 2, 0)]


@pytest.mark.parametrize("R,stride,pad", CONV_CASES)
def test_conv_finite_differences(R, stride, pad):
    N, Ci, Co, H, W = 2, 3, 2, 5, 4
    x = RNG.standard_normal((N, Ci, H, W))
    w = RNG.standard_normal((Co, Ci, R, R))
    y = orc.conv_fwd(x, w, stride, pad)
    r = RNG.standard_normal(y.shape)
    dx = orc.conv_bwd_data(r, w, (H, W), stride, pad)
    dw = orc.conv_bwd_weight(x, r, R, stride, pad)
    gx = fd_grad(lambda xx: float((orc.conv_fwd(xx, w, stride, pad) * r).sum()), x.copy())
    gw = fd_grad(lambda ww: float((orc.conv_fwd(x, ww, stride, pad) * r).sum()), w.copy())
    np.testing.assert_allclose(dx, gx, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dw, gw, rtol=1e-6, atol=1e-8)


@pytest.mark.parametrize("R,stride,pad", CONV_CASES)
def test_conv_adjoint_identities(R, stride, pad):
    N, Ci, Co, H, W = 3, 5, 4, 9, 7
    x = RNG.standard_normal((N, Ci, H, W))
    w = RNG.standard_normal((Co, Ci, R, R))
    y = orc.conv_fwd(x, w, stride, pad)
    d = RNG.standard_normal(y.shape)
    lhs = float((y * d).sum())
    assert abs(lhs - float((x * orc.conv_bwd_data(d, w, (H, W), stride, pad)).sum())) < 1e-9 * max(1, abs(lhs))
    assert abs(lhs - float((w * orc.conv_bwd_weight(x, d, R, stride, pad)).sum())) < 1e-9 * max(1, abs(lhs))


def test_conv_1x1_is_matrix_product():
    N, Ci, Co, H, W = 2, 6, 5, 4, 3
    x = RNG.standard_normal((N, Ci, H, W))
    w = RNG.standard_normal((Co, Ci, 1, 1))
    y = orc.conv_fwd(x, w, 1, 0)
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    y2 = orc.conv_fwd(x, w, 2, 0)
    np.testing.assert_allclose(y2, ref[:, :, ::2, ::2], rtol=1e-12, atol=1e-12)


def test_conv_centre_tap_is_identity_and_shift():
    N, C_, H, W = 2, 3, 6, 5
    x = RNG.standard_normal((N, C_, H, W))
    w = np.zeros((C_, C_, 3, 3))
    for c in range(C_):
        w[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(orc.conv_fwd(x, w), x)
    # tap (r=0, s=2) reads x[p-1, q+1]: a transposed or flipped kernel index would fail
    w2 = np.zeros((1, C_, 3, 3))
    w2[0, 1, 0, 2] = 1.0
    y = orc.conv_fwd(x, w2)
    ref = np.zeros((N, 1, H, W))
    ref[:, 0, 1:, :-1] = x[:, 1, :-1, 1:]
    np.testing.assert_array_equal(y, ref)


def test_conv_ones_counts_padding():
    Ci = 3
    x = np.ones((1, Ci, 5, 6))
    w = np.ones((2, Ci, 3, 3))
    y = orc.conv_fwd(x, w)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * Ci)
    assert np.all(y[:, :, 0, 1:-1] == 6 * Ci) and np.all(y[:, :, 1:-1, 0] == 6 * Ci)
    for p, q in ((0, 0), (0, -1), (-1, 0), (-1, -1)):
        assert np.all(y[:, :, p, q] == 4 * Ci)


def test_conv_matches_torch_fp64():
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    for R, stride, pad in CONV_CASES:
        x = RNG.standard_normal((2, 4, 8, 7))
        w = RNG.standard_normal((5, 4, R, R))
        y = orc.conv_fwd(x, w, stride, pad)
        ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=stride, padding=pad).numpy()
        np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_bn_forward_identities():
    N, C_, H, W = 4, 3, 5, 6
    x = 2.0 * RNG.standard_normal((N, C_, H, W)) + 0.7
    gamma = RNG.standard_normal(C_) + 1.5
    beta = RNG.standard_normal(C_)
    eps = 1e-5
    y, mean, invstd = orc.bn_fwd(x, gamma, beta, eps)
    xm = x.transpose(1, 0, 2, 3).reshape(C_, -1)
    np.testing.assert_allclose(mean, xm.mean(1), rtol=1e-12)
    var = xm.var(1)  # biased
    np.testing.assert_allclose(invstd, 1 / np.sqrt(var + eps), rtol=1e-12)
    ym = y.transpose(1, 0, 2, 3).reshape(C_, -1)
    np.testing.assert_allclose(ym.mean(1), beta, atol=1e-12)
    np.testing.assert_allclose(ym.var(1), gamma ** 2 * var / (var + eps), rtol=1e-10)


def test_bn_backward_finite_differences_and_identities():
    N, C_, H, W = 2, 3, 4, 4
    x = RNG.standard_normal((N, C_, H, W))
    gamma = RNG.standard_normal(C_) + 1.5
    beta = RNG.standard_normal(C_)
    r = RNG.standard_normal(x.shape)
    eps = 1e-5
    y, mean, invstd = orc.bn_fwd(x, gamma, beta, eps)
    dx, dg, db = orc.bn_bwd(r, x, mean, invstd, gamma)
    f = lambda xx, gg, bb: float((orc.bn_fwd(xx, gg, bb, eps)[0] * r).sum())
    np.testing.assert_allclose(dx, fd_grad(lambda v: f(v, gamma, beta), x.copy()), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dg, fd_grad(lambda v: f(x, v, beta), gamma.copy()), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db, fd_grad(lambda v: f(x, gamma, v), beta.copy()), rtol=1e-6, atol=1e-8)
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    assert np.abs(dx.sum((0, 2, 3))).max() < 1e-12
    # sum dx*xhat = gamma*invstd*dgamma*(1 - sum(xhat^2)/m), which is 0 only as eps -> 0
    m = N * H * W
    expect = gamma * invstd * dg * (1 - (xhat ** 2).sum((0, 2, 3)) / m)
    np.testing.assert_allclose((dx * xhat).sum((0, 2, 3)), expect, atol=1e-12)
    y0, mean0, invstd0 = orc.bn_fwd(x, gamma, beta, 0.0)
    dx0, _, _ = orc.bn_bwd(r, x, mean0, invstd0, gamma)
    xhat0 = (x - mean0[None, :, None, None]) * invstd0[None, :, None, None]
    assert np.abs((dx0 * xhat0).sum((0, 2, 3))).max() < 1e-12


def test_conv_then_bn_is_scale_invariant():
    """BN removes the scale of each filter, so <W_co, dW_co> vanishes as eps -> 0."""
    N, Ci, Co, H, W = 3, 4, 5, 6, 6
    x = RNG.standard_normal((N, Ci, H, W))
    w = RNG.standard_normal((Co, Ci, 3, 3))
    gamma, beta = RNG.standard_normal(Co) + 1.5, RNG.standard_normal(Co)
    z = orc.conv_fwd(x, w)
    y, mean, invstd = orc.bn_fwd(z, gamma, beta, 1e-12)
    r = RNG.standard_normal(y.shape)
    dz, _, _ = orc.bn_bwd(r, z, mean, invstd, gamma)
    dw = orc.conv_bwd_weight(x, dz, 3)
    inner = (w * dw).sum((1, 2, 3))
    assert np.abs(inner).max() < 1e-8 * np.abs(dw).max() * np.abs(w).max() * w[0].size


def test_head_closed_forms_and_finite_differences():
    N, C_, H, W, classes = 4, 5, 3, 3, 10
    h = RNG.standard_normal((N, C_, H, W))
    labels = np.array([3, 0, 9, 3], np.int32)
    loss, logits, dh, dw, db = orc.head(h, np.zeros((classes, C_)), np.zeros(classes), labels)
    assert abs(loss - 2.302585092994046) < 1e-12          # ln 10
    loss100, *_ = orc.head(h, np.zeros((100, C_)), np.zeros(100), labels)
    assert abs(loss100 - 4.605170185988092) < 1e-12       # ln 100
    fcw = RNG.standard_normal((classes, C_))
    fcb = RNG.standard_normal(classes)
    loss, logits, dh, dw, db = orc.head(h, fcw, fcb, labels)
    pooled = h.mean((2, 3))
    np.testing.assert_allclose(logits, pooled @ fcw.T + fcb, rtol=1e-12)
    # softmax - onehot rows sum to zero => db sums to zero
    assert abs(db.sum()) < 1e-12
    f = lambda hh, ww, bb: orc.head(hh, ww, bb, labels, want_grads=False)[0]
    np.testing.assert_allclose(dh, fd_grad(lambda v: f(v, fcw, fcb), h.copy()), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(dw, fd_grad(lambda v: f(h, v, fcb), fcw.copy()), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(db, fd_grad(lambda v: f(h, fcw, v), fcb.copy()), rtol=1e-6, atol=1e-9)
    # very large logits: the stable softmax must not overflow
    big, *_ = orc.head(h, 1e3 * fcw, fcb, labels, want_grads=False)
    assert np.isfinite(big)


def test_float32_instance_agrees_with_float64():
    x = RNG.standard_normal((2, 4, 8, 8))
    w = RNG.standard_normal((6, 4, 3, 3))
    y64 = orc.conv_fwd(x, w)
    y32 = orc.conv_fwd(x, w, dtype="f32")
    assert y32.dtype == np.float32
    np.testing.assert_allclose(y32, y64, rtol=1e-4, atol=1e-4)
