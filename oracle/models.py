"""The networks of the measured workloads, forward and backward, in float64.

MLP: 3072 -> 128 (ReLU) -> 10 on flattened images.  ResNetCifar: the CIFAR residual network of
He et al. (2016) that the paper calls ResNet20 (Section 5): 3x3 stem, 3 stages x 3 basic blocks
of widths 16/32/64, parameter-free shortcuts, global average pooling and a linear classifier.
Widths, depth and image size are arguments so that tiny instances can be checked by finite
differences.  Parameters and buffers are dicts of float64 arrays keyed by tensor name.

Mixed precision.  ResNetCifar takes an optional `storage` function (e.g. precision.round_bf16)
that maps an array onto the grid of the format activations are kept in.  It is applied wherever a
mixed-precision run holds a tensor in that format: the input images, the convolution weights as the
convolutions read them (the parameters themselves stay full precision), every convolution output
that batch norm takes its batch statistics from, every activation, and in the backward pass every
gradient with respect to a convolution output or a convolution input.  Sums, statistics, the
classifier, losses and parameter gradients are never rounded.  With storage=None (the default) this
is the plain float64 model.
"""
import numpy as np

from . import layers as L


def _f64(d):
    return {k: np.asarray(v, dtype=np.float64) for k, v in d.items()}


class MLP:
    has_buffers = False

    def forward(self, params, buffers, x, train):
        p = _f64(params)
        x2 = np.asarray(x, dtype=np.float64).reshape(x.shape[0], -1)
        h = L.relu(L.linear(x2, p["fc1.weight"], p["fc1.bias"]))
        logits = L.linear(h, p["fc2.weight"], p["fc2.bias"])
        return logits, (p, x2, h), dict(buffers)

    def backward(self, cache, dlogits):
        p, x2, h = cache
        dh, dw2, db2 = L.linear_backward(h, p["fc2.weight"], dlogits)
        dpre = L.relu_backward(dh, h)
        _, dw1, db1 = L.linear_backward(x2, p["fc1.weight"], dpre)
        return {"fc1.weight": dw1, "fc1.bias": db1, "fc2.weight": dw2, "fc2.bias": db2}


class ResNetCifar:
    has_buffers = True

    def __init__(self, widths=(16, 32, 64), blocks=3, storage=None):
        self.widths = tuple(widths)
        self.blocks = blocks
        self.q = storage if storage is not None else (lambda a: a)

    def _block_list(self):
        out, c_prev = [], self.widths[0]
        for s, c in enumerate(self.widths):
            for b in range(self.blocks):
                out.append(("s%d.b%d" % (s + 1, b), c_prev, c, 2 if (b == 0 and s > 0) else 1))
                c_prev = c
        return out

    def _bn(self, name, x, p, bufs, new_bufs, train):
        g, b = p[name + ".weight"], p[name + ".bias"]
        rm, rv = bufs[name + ".running_mean"], bufs[name + ".running_var"]
        if not train:
            return L.batchnorm_eval(x, g, b, rm, rv), None
        y, cache, nrm, nrv = L.batchnorm_train(x, g, b, rm, rv)
        new_bufs[name + ".running_mean"], new_bufs[name + ".running_var"] = nrm, nrv
        return y, cache

    def forward(self, params, buffers, x, train):
        """Returns (logits [B, classes], cache for backward, buffers after this pass)."""
        p, bufs = _f64(params), _f64(buffers)
        q = self.q
        qy = q if train else (lambda a: a)   # in inference batch norm is applied to the unrounded convolution result
        # "w": the convolution weights as the convolutions read them
        cache_w = {k: q(v) for k, v in p.items() if k.endswith("conv.weight") or ".conv1." in k or ".conv2." in k}
        new_bufs = dict(bufs)
        x = q(np.asarray(x, dtype=np.float64))
        cache = {"p": p, "w": cache_w, "x": x, "z": {}}   # "z": pre-activation of every ReLU, keyed by the name of its output
        w = cache_w
        y0 = qy(L.conv3x3(x, w["stem.conv.weight"], 1))
        z0, cache["stem.bn"] = self._bn("stem.bn", y0, p, bufs, new_bufs, train)
        cache["z"]["stem.out"] = z0
        a = q(L.relu(z0))
        cache["stem.out"] = a
        for name, c_in, c_out, stride in self._block_list():
            cache[name + ".in"] = a
            y1 = qy(L.conv3x3(a, w[name + ".conv1.weight"], stride))
            z1, cache[name + ".bn1"] = self._bn(name + ".bn1", y1, p, bufs, new_bufs, train)
            cache["z"][name + ".h1"] = z1
            h1 = q(L.relu(z1))
            cache[name + ".h1"] = h1
            y2 = qy(L.conv3x3(h1, w[name + ".conv2.weight"], 1))
            z2, cache[name + ".bn2"] = self._bn(name + ".bn2", y2, p, bufs, new_bufs, train)
            zo = z2 + L.shortcut(a, c_out, stride)
            cache["z"][name + ".out"] = zo
            a = q(L.relu(zo))
            cache[name + ".out"] = a
        cache["final"] = a
        pooled = L.global_avgpool(a)
        cache["pooled"] = pooled
        logits = L.linear(pooled, p["fc.weight"], p["fc.bias"])
        return logits, cache, new_bufs

    def backward(self, cache, dlogits, toggles=None):
        """Gradients of sum_b <dlogits_b, logits_b> with respect to every parameter (train mode).

        toggles: optional {relu output name: flat indices} passed to relu_backward."""
        p, w, q = cache["p"], cache["w"], self.q
        g = {}
        tg = toggles or {}
        dpooled, g["fc.weight"], g["fc.bias"] = L.linear_backward(cache["pooled"], p["fc.weight"], dlogits)
        da = L.global_avgpool_backward(dpooled, cache["final"].shape)
        for name, c_in, c_out, stride in reversed(self._block_list()):
            dz = L.relu_backward(da, cache[name + ".out"], tg.get(name + ".out"))
            dy2, g[name + ".bn2.weight"], g[name + ".bn2.bias"] = L.batchnorm_train_backward(dz, cache[name + ".bn2"])
            dy2 = q(dy2)
            dh1, g[name + ".conv2.weight"] = L.conv3x3_backward(cache[name + ".h1"], w[name + ".conv2.weight"], dy2, 1)
            dz1 = L.relu_backward(q(dh1), cache[name + ".h1"], tg.get(name + ".h1"))
            dy1, g[name + ".bn1.weight"], g[name + ".bn1.bias"] = L.batchnorm_train_backward(dz1, cache[name + ".bn1"])
            dy1 = q(dy1)
            x_in = cache[name + ".in"]
            dx, g[name + ".conv1.weight"] = L.conv3x3_backward(x_in, w[name + ".conv1.weight"], dy1, stride)
            da = q(dx + L.shortcut_backward(q(dz), x_in.shape, stride))
        dz0 = L.relu_backward(da, cache["stem.out"], tg.get("stem.out"))
        dy0, g["stem.bn.weight"], g["stem.bn.bias"] = L.batchnorm_train_backward(dz0, cache["stem.bn"])
        _, g["stem.conv.weight"] = L.conv3x3_backward(cache["x"], w["stem.conv.weight"], q(dy0), 1, need_dx=False)
        return g


class WideResNet:
    """Wide residual network for 32x32 images (Zagoruyko & Komodakis 2016), the WRN16 family of Section 5.

    Depth 6 * blocks + 4 with widening factor widths[0] / 16: a 3x3 stem to `stem` channels, three stages of
    `blocks` pre-activation blocks  out = shortcut + conv2(relu(bn2(conv1(relu(bn1(x))))))  where the first
    block of stages 2 and 3 has stride 2, and the shortcut is the identity when the block keeps its shape
    and otherwise a 1x1 convolution (same stride) of relu(bn1(x)); then batch norm, ReLU, global average
    pooling and a linear classifier.  WRN-16-8 is widths (128, 256, 512), blocks 2, stem 16.
    `storage` has the meaning described at the top of this file.
    """
    has_buffers = True

    def __init__(self, widths=(128, 256, 512), blocks=2, stem=16, storage=None):
        self.widths, self.blocks, self.stem = tuple(widths), blocks, stem
        self.q = storage if storage is not None else (lambda a: a)

    def block_list(self):
        out, c_prev = [], self.stem
        for s, c in enumerate(self.widths):
            for b in range(self.blocks):
                stride = 2 if (b == 0 and s > 0) else 1
                out.append(("s%d.b%d" % (s + 1, b), c_prev, c, stride, c_prev != c or stride != 1))
                c_prev = c
        return out

    def _bn(self, name, x, p, bufs, new_bufs, train):
        g, b = p[name + ".weight"], p[name + ".bias"]
        rm, rv = bufs[name + ".running_mean"], bufs[name + ".running_var"]
        if not train:
            return L.batchnorm_eval(x, g, b, rm, rv), None
        y, cache, nrm, nrv = L.batchnorm_train(x, g, b, rm, rv)
        new_bufs[name + ".running_mean"], new_bufs[name + ".running_var"] = nrm, nrv
        return y, cache

    def forward(self, params, buffers, x, train):
        p, bufs = _f64(params), _f64(buffers)
        q = self.q
        w = {k: q(v) for k, v in p.items() if k.endswith("conv.weight") or ".conv1." in k or ".conv2." in k or ".shortcut." in k}
        new_bufs = dict(bufs)
        x = q(np.asarray(x, dtype=np.float64))
        cache = {"p": p, "w": w, "x": x, "z": {}}
        cur = q(L.conv3x3(x, w["stem.conv.weight"], 1))
        for name, c_in, c_out, stride, proj in self.block_list():
            cache[name + ".in"] = cur
            z1, cache[name + ".bn1"] = self._bn(name + ".bn1", cur, p, bufs, new_bufs, train)
            cache["z"][name + ".o1"] = z1
            o1 = q(L.relu(z1))
            cache[name + ".o1"] = o1
            y1 = q(L.conv3x3(o1, w[name + ".conv1.weight"], stride))
            z2, cache[name + ".bn2"] = self._bn(name + ".bn2", y1, p, bufs, new_bufs, train)
            cache["z"][name + ".o2"] = z2
            o2 = q(L.relu(z2))
            cache[name + ".o2"] = o2
            sc = q(L.conv1x1(o1, w[name + ".shortcut.weight"], stride)) if proj else cur
            cur = q(L.conv3x3(o2, w[name + ".conv2.weight"], 1) + sc)
        cache["last"] = cur
        zf, cache["final.bn"] = self._bn("final.bn", cur, p, bufs, new_bufs, train)
        cache["z"]["final"] = zf
        a = q(L.relu(zf))
        cache["final"] = a
        pooled = L.global_avgpool(a)
        cache["pooled"] = pooled
        logits = L.linear(pooled, p["fc.weight"], p["fc.bias"])
        return logits, cache, new_bufs

    def backward(self, cache, dlogits, toggles=None):
        p, w, q = cache["p"], cache["w"], self.q
        g, tg = {}, toggles or {}
        dpooled, g["fc.weight"], g["fc.bias"] = L.linear_backward(cache["pooled"], p["fc.weight"], dlogits)
        da = L.global_avgpool_backward(dpooled, cache["final"].shape)
        dzf = L.relu_backward(da, cache["final"], tg.get("final"))
        dout, g["final.bn.weight"], g["final.bn.bias"] = L.batchnorm_train_backward(dzf, cache["final.bn"])
        dout = q(dout)
        for name, c_in, c_out, stride, proj in reversed(self.block_list()):
            o1, o2 = cache[name + ".o1"], cache[name + ".o2"]
            do2, g[name + ".conv2.weight"] = L.conv3x3_backward(o2, w[name + ".conv2.weight"], dout, 1)
            dz2 = L.relu_backward(q(do2), o2, tg.get(name + ".o2"))
            dy1, g[name + ".bn2.weight"], g[name + ".bn2.bias"] = L.batchnorm_train_backward(dz2, cache[name + ".bn2"])
            dy1 = q(dy1)
            do1, g[name + ".conv1.weight"] = L.conv3x3_backward(o1, w[name + ".conv1.weight"], dy1, stride)
            if proj:
                dsc, g[name + ".shortcut.weight"] = L.conv1x1_backward(o1, w[name + ".shortcut.weight"], dout, stride)
                do1 = do1 + q(dsc)
            dz1 = L.relu_backward(q(do1), o1, tg.get(name + ".o1"))
            dx, g[name + ".bn1.weight"], g[name + ".bn1.bias"] = L.batchnorm_train_backward(dz1, cache[name + ".bn1"])
            dout = q(dx if proj else dx + dout)
        _, g["stem.conv.weight"] = L.conv3x3_backward(cache["x"], w["stem.conv.weight"], dout, 1, need_dx=False)
        return g
