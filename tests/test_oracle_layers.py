"""Pins for the oracle's layers: brute force, library special cases, invariants, finite differences."""
import numpy as np
import pytest
from scipy.signal import correlate2d
from scipy.special import logsumexp

import synth
from oracle import layers as L
from oracle.losses import softmax_cross_entropy


def _rand(stream, *shape):
    return synth.normal(77, stream, int(np.prod(shape))).reshape(shape)


def _fd(f, x, eps=1e-6):
    """Central finite-difference gradient of scalar f at x (float64)."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = f()
        x[i] = old - eps
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def _conv_loops(x, w, stride):
    n, H, W, ci = x.shape
    co = w.shape[0]
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    out = np.zeros((n, Ho, Wo, co))
    for b in range(n):
        for h in range(Ho):
            for ww in range(Wo):
                for o in range(co):
                    acc = 0.0
                    for kh in range(3):
                        for kw in range(3):
                            hi, wi = stride * h + kh - 1, stride * ww + kw - 1
                            if 0 <= hi < H and 0 <= wi < W:
                                for i in range(ci):
                                    acc += x[b, hi, wi, i] * w[o, kh, kw, i]
                    out[b, h, ww, o] = acc
    return out


@pytest.mark.parametrize("stride,H,W", [(1, 5, 6), (2, 6, 8), (2, 5, 7)])
def test_conv_against_nested_loops(stride, H, W):
    x, w = _rand(1, 2, H, W, 3), _rand(2, 4, 3, 3, 3)
    np.testing.assert_allclose(L.conv3x3(x, w, stride), _conv_loops(x, w, stride), rtol=1e-12, atol=1e-12)


def test_conv_library_special_case_and_delta_kernel():
    x, w = _rand(3, 1, 9, 7, 1), _rand(4, 1, 3, 3, 1)
    ref = correlate2d(x[0, :, :, 0], w[0, :, :, 0], mode="same", boundary="fill")
    np.testing.assert_allclose(L.conv3x3(x, w, 1)[0, :, :, 0], ref, rtol=1e-12, atol=1e-12)
    x = _rand(5, 2, 6, 6, 4)
    delta = np.zeros((4, 3, 3, 4))
    for c in range(4):
        delta[c, 1, 1, c] = 1.0
    np.testing.assert_array_equal(L.conv3x3(x, delta, 1), x)
    # stride 2 keeps every second output of the stride-1 result
    w = _rand(6, 5, 3, 3, 4)
    np.testing.assert_allclose(L.conv3x3(x, w, 2), L.conv3x3(x, w, 1)[:, ::2, ::2, :], rtol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
def test_conv_backward_finite_differences(stride):
    x, w = _rand(7, 2, 6, 6, 3), _rand(8, 4, 3, 3, 3)
    r = _rand(9, *L.conv3x3(x, w, stride).shape)
    f = lambda: float((L.conv3x3(x, w, stride) * r).sum())
    dx, dw = L.conv3x3_backward(x, w, r, stride)
    np.testing.assert_allclose(dx, _fd(f, x), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dw, _fd(f, w), rtol=1e-6, atol=1e-7)


def test_batchnorm_train_invariants():
    x = 3.0 + 2.0 * _rand(10, 8, 4, 4, 5)
    g, b = _rand(11, 5), _rand(12, 5)
    y, _, rm, rv = L.batchnorm_train(x, g, b, np.zeros(5), np.ones(5))
    xf = x.reshape(-1, 5)
    yhat = (y - b) / g
    np.testing.assert_allclose(yhat.reshape(-1, 5).mean(axis=0), 0, atol=1e-12)
    np.testing.assert_allclose((yhat ** 2).reshape(-1, 5).mean(axis=0), xf.var(axis=0) / (xf.var(axis=0) + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(rm, 0.1 * xf.mean(axis=0), rtol=1e-12)
    np.testing.assert_allclose(rv, 0.9 + 0.1 * xf.var(axis=0, ddof=1), rtol=1e-12)
    # a constant batch normalises to the shift
    yc, _, _, _ = L.batchnorm_train(np.full((4, 2, 2, 5), 7.0), g, b, np.zeros(5), np.ones(5))
    np.testing.assert_allclose(yc, np.broadcast_to(b, yc.shape), atol=1e-12)


def test_batchnorm_eval_closed_form():
    x = _rand(13, 3, 2, 2, 4)
    g, b, rm, rv = _rand(14, 4), _rand(15, 4), _rand(16, 4), 1.0 + np.abs(_rand(17, 4))
    np.testing.assert_allclose(L.batchnorm_eval(x, g, b, np.zeros(4), np.ones(4)), g * x / np.sqrt(1 + 1e-5) + b, rtol=1e-13)
    y = L.batchnorm_eval(x, g, b, rm, rv)
    np.testing.assert_allclose((y - b) / g * np.sqrt(rv + 1e-5) + rm, x, rtol=1e-11, atol=1e-12)


def test_batchnorm_backward_finite_differences():
    x, g, b = _rand(18, 4, 3, 3, 2), 1.0 + 0.3 * _rand(19, 2), _rand(20, 2)
    r = _rand(21, 4, 3, 3, 2)
    f = lambda: float((L.batchnorm_train(x, g, b, np.zeros(2), np.ones(2))[0] * r).sum())
    _, cache, _, _ = L.batchnorm_train(x, g, b, np.zeros(2), np.ones(2))
    dx, dg, db = L.batchnorm_train_backward(r, cache)
    np.testing.assert_allclose(dx, _fd(f, x), rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(dg, _fd(f, g), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(db, _fd(f, b), rtol=1e-6, atol=1e-7)


def test_cross_entropy_pins():
    for C in (10, 100, 32000):
        loss, d = softmax_cross_entropy(np.zeros((3, C)), [0, C // 2, C - 1])
        np.testing.assert_allclose(loss, np.log(C), rtol=1e-14)
    z = _rand(22, 6, 10) * 3
    y = np.array([0, 3, 9, 9, 1, 5])
    loss, d = softmax_cross_entropy(z, y)
    np.testing.assert_allclose(loss, logsumexp(z, axis=1) - z[np.arange(6), y], rtol=1e-13)
    np.testing.assert_allclose(softmax_cross_entropy(z + 123.0, y)[0], loss, rtol=1e-10)
    np.testing.assert_allclose(d.sum(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose((d + np.eye(10)[y]).sum(axis=1), 1.0, rtol=1e-14)
    big = np.array([[1e4, -1e4, 0.0], [-1e4, 1e4, 0.0]])
    lb, _ = softmax_cross_entropy(big, [0, 0])
    assert np.all(np.isfinite(lb)) and abs(lb[0]) < 1e-12 and abs(lb[1] - 2e4) < 1e-8
    f = lambda: float(softmax_cross_entropy(z, y)[0].sum())
    np.testing.assert_allclose(d, _fd(f, z), rtol=1e-6, atol=1e-8)


def test_shortcut_pool_linear_relu():
    x = _rand(23, 2, 4, 4, 2)
    s = L.shortcut(x, 4, 2)
    assert s.shape == (2, 2, 2, 4)
    np.testing.assert_array_equal(s[..., 1:3], x[:, ::2, ::2, :])
    assert np.all(s[..., 0] == 0) and np.all(s[..., 3] == 0)
    assert L.shortcut(x, 2, 1) is x
    r = _rand(24, 2, 2, 2, 4)
    f = lambda: float((L.shortcut(x, 4, 2) * r).sum())
    np.testing.assert_allclose(L.shortcut_backward(r, x.shape, 2), _fd(f, x), atol=1e-8)
    np.testing.assert_allclose(L.global_avgpool(x), x.reshape(2, 16, 2).mean(axis=1), rtol=1e-14)
    rp = _rand(25, 2, 2)
    f = lambda: float((L.global_avgpool(x) * rp).sum())
    np.testing.assert_allclose(L.global_avgpool_backward(rp, x.shape), _fd(f, x), atol=1e-8)
    a, w, b = _rand(26, 3, 5), _rand(27, 4, 5), _rand(28, 4)
    np.testing.assert_allclose(L.linear(a, w, b), np.einsum("bi,oi->bo", a, w) + b, rtol=1e-13)
    ry = _rand(29, 3, 4)
    f = lambda: float((L.linear(a, w, b) * ry).sum())
    da, dw, db = L.linear_backward(a, w, ry)
    np.testing.assert_allclose(da, _fd(f, a), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dw, _fd(f, w), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db, _fd(f, b), rtol=1e-6, atol=1e-8)
    v = np.array([-1.0, 0.0, 2.0])
    np.testing.assert_array_equal(L.relu(v), [0, 0, 2])
    np.testing.assert_array_equal(L.relu_backward(np.ones(3), L.relu(v)), [0, 0, 1])
