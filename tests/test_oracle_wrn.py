"""Pins of the wide residual network in the oracle: parameter counts of WRN-16-8 worked by hand,
finite-difference gradients on a tiny instance, the 1x1 projection against its definition, and
reductions to known special cases."""
import numpy as np

import oracle
import synth
from oracle import layers as L


def test_wrn16_8_parameter_counts():
    # by hand: stem 3*16*9 = 432; stage 1: 16*128*9 + 3 * 128*128*9 + 16*128 = 462 848; stage 2: 128*256*9 +
    # 3 * 256*256*9 + 128*256 = 2 097 152; stage 3: 256*512*9 + 3 * 512*512*9 + 256*512 = 8 388 608;
    # batch norm: channels 16+128, 128+128, 128+256, 256+256, 256+512, 512+512, 512 = 3600, two vectors each;
    # classifier 512*100 + 100
    ps, bs = synth.wrn_tensor_specs()
    convs = sum(int(np.prod(s)) for n, s in ps if len(s) == 4)
    bn = sum(int(np.prod(s)) for n, s in ps if len(s) == 1 and not n.startswith("fc"))
    fc = sum(int(np.prod(s)) for n, s in ps if n.startswith("fc"))
    assert (convs, bn, fc) == (432 + 462848 + 2097152 + 8388608, 7200, 51300)
    assert convs + bn + fc == 11007540
    assert sum(int(np.prod(s)) for n, s in bs) == 7200
    assert [n for n, s in ps if "shortcut" in n] == ["s1.b0.shortcut.weight", "s2.b0.shortcut.weight", "s3.b0.shortcut.weight"]


def test_conv1x1_is_a_strided_channel_mix():
    rs = np.random.RandomState(0)
    x = rs.standard_normal((2, 4, 4, 3))
    w = rs.standard_normal((5, 1, 1, 3))
    out = L.conv1x1(x, w, 2)
    assert out.shape == (2, 2, 2, 5)
    for n in range(2):
        for h in range(2):
            for v in range(2):
                np.testing.assert_allclose(out[n, h, v], w[:, 0, 0, :] @ x[n, 2 * h, 2 * v], rtol=1e-13)
    # adjoint identities <dout, conv(x)> = <dx, x> = <dw, w>
    dout = rs.standard_normal(out.shape)
    dx, dw = L.conv1x1_backward(x, w, dout, 2)
    np.testing.assert_allclose((dout * out).sum(), (dx * x).sum(), rtol=1e-12)
    np.testing.assert_allclose((dout * out).sum(), (dw * w).sum(), rtol=1e-12)
    # a 1x1 convolution equals a 3x3 one whose only non-zero tap is the centre
    w3 = np.zeros((5, 3, 3, 3))
    w3[:, 1, 1, :] = w[:, 0, 0, :]
    np.testing.assert_allclose(L.conv3x3(x, w3, 2), out, rtol=1e-13, atol=1e-13)


def _tiny():
    widths, stem = (4, 4, 6), 2          # stage 2 keeps the width (identity shortcut only when the stride is 1)
    model = oracle.WideResNet(widths, blocks=2, stem=stem)
    p, b = synth.wrn_init(5, widths, 2, classes=3, stem=stem, perturb_bn=0.3)
    x, y = synth.image_pool(5, 5, 3, hw=8)
    return model, {k: v.astype(np.float64) for k, v in p.items()}, b, x.astype(np.float64), y


def test_gradients_finite_differences():
    model, p, b, x, y = _tiny()
    losses, grads, _ = oracle.loss_and_grads(model, p, b, x, y)
    assert set(grads) == set(p)
    eps = 1e-6
    for name, t in p.items():
        flat = t.reshape(-1)
        picks = range(flat.size) if flat.size <= 12 else synth.randint(6, len(name), 12, flat.size)
        for i in picks:
            old = flat[i]
            flat[i] = old + eps
            lp = oracle.loss_and_grads(model, p, b, x, y)[0].mean()
            flat[i] = old - eps
            lm = oracle.loss_and_grads(model, p, b, x, y)[0].mean()
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grads[name].reshape(-1)[i]) <= 3e-5 * max(1e-3, abs(fd)), (name, i, fd, grads[name].reshape(-1)[i])


def test_structure():
    model, p, b, x, y = _tiny()
    blocks = model.block_list()
    assert [(n, s, pr) for n, ci, co, s, pr in blocks] == [("s1.b0", 1, True), ("s1.b1", 1, False), ("s2.b0", 2, True),
                                                          ("s2.b1", 1, False), ("s3.b0", 2, True), ("s3.b1", 1, False)]
    logits, cache, nb = model.forward(p, b, x, train=True)
    assert logits.shape == (5, 3) and cache["last"].shape == (5, 2, 2, 6)
    # identity blocks: zero convolutions make the block the identity
    p2 = {k: v.copy() for k, v in p.items()}
    p2["s1.b1.conv2.weight"][:] = 0
    _, c2, _ = model.forward(p2, b, x, train=True)
    np.testing.assert_array_equal(c2["s2.b0.in"], c2["s1.b1.in"])
    # a zero classifier gives ln(classes) for every sample, in both modes
    p2["fc.weight"][:] = 0
    p2["fc.bias"][:] = 0
    np.testing.assert_allclose(oracle.score_losses(model, p2, b, x, y), np.log(3.0), rtol=1e-14)
    # inference uses running statistics: a score does not depend on the rest of the pool
    s_all = oracle.score_losses(model, p, b, x, y)
    np.testing.assert_allclose(oracle.score_losses(model, p, b, x[1:3], y[1:3]), s_all[1:3], rtol=1e-12)
    # running statistics move for every batch norm in training
    assert all(not np.array_equal(nb[k], np.asarray(b[k], np.float64)) for k in nb)


def test_storage_hook_identity_and_rounding():
    model, p, b, x, y = _tiny()
    calls = []
    hooked = oracle.WideResNet(model.widths, model.blocks, model.stem, storage=lambda a: (calls.append(1), a)[1])
    l0, g0, _ = oracle.loss_and_grads(model, p, b, x, y)
    l1, g1, _ = oracle.loss_and_grads(hooked, p, b, x, y)
    np.testing.assert_array_equal(l0, l1)
    for k in g0:
        np.testing.assert_array_equal(g0[k], g1[k])
    rounded = oracle.WideResNet(model.widths, model.blocks, model.stem, storage=oracle.round_bf16)
    _, cache, _ = rounded.forward(p, b, x, train=True)
    for name in ["x", "s1.b0.o1", "s1.b0.o2", "s2.b0.in", "last", "final"]:
        np.testing.assert_array_equal(cache[name], oracle.round_bf16(cache[name]))
