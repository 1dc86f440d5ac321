"""Layer definitions (forward and hand-derived backward) in float64, NHWC.

These are the textbook building blocks of the networks the paper trains (ResNet20 on
CIFAR-10, Section 5): 3x3 convolution with zero padding 1, training- and inference-mode
batch normalisation, ReLU, global average pooling and a linear layer, plus the 1x1 projection of the
wide residual networks (WRN16, Section 5).  Convolution weights are [C_out, kh, kw, C_in]; images are
[N, H, W, C].
"""
import numpy as np

BN_EPS = 1e-5
BN_MOMENTUM = 0.1


def conv3x3(x, w, stride=1):
    """out[n,h,w,o] = sum_{kh,kw,i} xpad[n, s*h+kh, s*w+kw, i] * w[o,kh,kw,i]  (padding 1)."""
    n, H, W, ci = x.shape
    co = w.shape[0]
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    xp = np.zeros((n, H + 2, W + 2, ci), dtype=np.float64)
    xp[:, 1:H + 1, 1:W + 1, :] = x
    out = np.zeros((n, Ho, Wo, co), dtype=np.float64)
    for kh in range(3):
        for kw in range(3):
            xs = xp[:, kh:kh + stride * (Ho - 1) + 1:stride, kw:kw + stride * (Wo - 1) + 1:stride, :]
            out += xs @ w[:, kh, kw, :].T
    return out


def conv3x3_backward(x, w, dout, stride=1, need_dx=True):
    """(dx, dw): adjoints of conv3x3 with respect to its input and its weights."""
    n, H, W, ci = x.shape
    Ho, Wo = dout.shape[1], dout.shape[2]
    xp = np.zeros((n, H + 2, W + 2, ci), dtype=np.float64)
    xp[:, 1:H + 1, 1:W + 1, :] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros(w.shape, dtype=np.float64)
    for kh in range(3):
        for kw in range(3):
            sl = (slice(None), slice(kh, kh + stride * (Ho - 1) + 1, stride),
                  slice(kw, kw + stride * (Wo - 1) + 1, stride), slice(None))
            dw[:, kh, kw, :] = np.tensordot(dout, xp[sl], axes=([0, 1, 2], [0, 1, 2]))
            if need_dx:
                dxp[sl] += dout @ w[:, kh, kw, :]
    return (dxp[:, 1:H + 1, 1:W + 1, :] if need_dx else None), dw


def conv1x1(x, w, stride=1):
    """out[n,h,w,o] = sum_i x[n, s*h, s*w, i] * w[o,0,0,i]: the projection shortcut of a residual block."""
    return x[:, ::stride, ::stride, :] @ w[:, 0, 0, :].T


def conv1x1_backward(x, w, dout, stride=1):
    """(dx, dw): adjoints of conv1x1."""
    dx = np.zeros(x.shape, dtype=np.float64)
    dx[:, ::stride, ::stride, :] = dout @ w[:, 0, 0, :]
    dw = np.tensordot(dout, x[:, ::stride, ::stride, :], axes=([0, 1, 2], [0, 1, 2])).reshape(w.shape)
    return dx, dw


def batchnorm_train(x, gamma, beta, running_mean, running_var):
    """Training-mode batch norm over (N, H, W).

    Normalises with the batch mean and the biased batch variance; the running statistics move
    by momentum 0.1 towards the batch mean and the unbiased batch variance.
    Returns (y, cache, new_running_mean, new_running_var).
    """
    c = x.shape[-1]
    xf = x.reshape(-1, c)
    m = xf.shape[0]
    mean = xf.mean(axis=0)
    var = ((xf - mean) ** 2).mean(axis=0)
    invstd = 1.0 / np.sqrt(var + BN_EPS)
    xhat = (x - mean) * invstd
    y = gamma * xhat + beta
    unbiased = var * m / (m - 1) if m > 1 else var
    new_rm = (1.0 - BN_MOMENTUM) * running_mean + BN_MOMENTUM * mean
    new_rv = (1.0 - BN_MOMENTUM) * running_var + BN_MOMENTUM * unbiased
    return y, (xhat, invstd, gamma), new_rm, new_rv


def batchnorm_train_backward(dy, cache):
    """(dx, dgamma, dbeta) of training-mode batch norm (the batch statistics depend on x)."""
    xhat, invstd, gamma = cache
    c = dy.shape[-1]
    m = dy.reshape(-1, c).shape[0]
    dbeta = dy.reshape(-1, c).sum(axis=0)
    dgamma = (dy * xhat).reshape(-1, c).sum(axis=0)
    dx = gamma * invstd * (dy - dbeta / m - xhat * (dgamma / m))
    return dx, dgamma, dbeta


def batchnorm_eval(x, gamma, beta, running_mean, running_var):
    """Inference-mode batch norm: a per-channel affine map from the running statistics."""
    return gamma * (x - running_mean) / np.sqrt(running_var + BN_EPS) + beta


def relu(x):
    return np.maximum(x, 0.0)


def relu_backward(dy, y, toggle=None):
    """ReLU'(0) = 0: the gradient passes only where the output is positive.

    `toggle` (flat indices) inverts the pass/block decision of those units.  It exists for
    comparisons with lower-precision implementations: where a pre-activation lies within rounding
    error of zero the two sides may legitimately land on different sides of the kink, and both
    one-sided derivatives are valid there.
    """
    mask = y > 0.0
    if toggle is not None and len(toggle):
        mask = mask.copy()
        flat = mask.reshape(-1)
        flat[np.asarray(toggle, dtype=np.int64)] ^= True
    return dy * mask


def shortcut(x, c_out, stride):
    """Identity, or the parameter-free shortcut of He et al. (2016) for CIFAR nets:
    spatial subsampling by `stride` and zero-padding of the extra channels on both sides."""
    c_in = x.shape[-1]
    if stride == 1 and c_in == c_out:
        return x
    xs = x[:, ::stride, ::stride, :]
    lo = (c_out - c_in) // 2
    out = np.zeros(xs.shape[:3] + (c_out,), dtype=np.float64)
    out[..., lo:lo + c_in] = xs
    return out


def shortcut_backward(dy, x_shape, stride):
    c_in, c_out = x_shape[-1], dy.shape[-1]
    if stride == 1 and c_in == c_out:
        return dy
    lo = (c_out - c_in) // 2
    dx = np.zeros(x_shape, dtype=np.float64)
    dx[:, ::stride, ::stride, :] = dy[..., lo:lo + c_in]
    return dx


def global_avgpool(x):
    return x.mean(axis=(1, 2))


def global_avgpool_backward(dy, x_shape):
    n, H, W, c = x_shape
    return np.broadcast_to(dy[:, None, None, :] / (H * W), x_shape).copy()


def linear(x, w, b):
    """y = x w^T + b with w [out, in]."""
    return x @ w.T + b


def linear_backward(x, w, dy):
    """(dx, dw, db)."""
    return dy @ w, dy.T @ x, dy.sum(axis=0)
