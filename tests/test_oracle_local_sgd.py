"""Pins for the oracle's networks, optimiser, scoring and local step."""
import numpy as np
import pytest

import oracle
import synth


def _tiny_resnet():
    widths = (2, 4, 8)
    model = oracle.ResNetCifar(widths, blocks=1)
    p, b = synth.resnet_init(3, widths, blocks=1, classes=3, perturb_bn=0.3)
    x, y = synth.image_pool(3, 6, 3, hw=8)
    return model, {k: v.astype(np.float64) for k, v in p.items()}, b, x.astype(np.float64), y


def _tiny_mlp(n=12, d_in=6, hidden=5, classes=3):
    p = synth.mlp_init(4, d_in, hidden, classes)
    x = synth.normal(4, 50, n * d_in).reshape(n, d_in)
    y = synth.randint(4, 51, n, classes).astype(np.int32)
    return oracle.MLP(), {k: v.astype(np.float64) for k, v in p.items()}, x, y


def _check_grads_fd(model, params, buffers, x, y, eps=1e-6, rtol=2e-5):
    losses, grads, _ = oracle.loss_and_grads(model, params, buffers, x, y)
    for name, t in params.items():
        flat = t.reshape(-1)
        picks = range(flat.size) if flat.size <= 40 else synth.randint(5, len(name), 40, flat.size)
        for i in picks:
            old = flat[i]
            flat[i] = old + eps
            lp = oracle.loss_and_grads(model, params, buffers, x, y)[0].mean()
            flat[i] = old - eps
            lm = oracle.loss_and_grads(model, params, buffers, x, y)[0].mean()
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grads[name].reshape(-1)[i]) <= rtol * max(1e-3, abs(fd)), (name, i, fd, grads[name].reshape(-1)[i])


def test_resnet_gradients_finite_differences():
    model, p, b, x, y = _tiny_resnet()
    _check_grads_fd(model, p, b, x, y)


def test_mlp_gradients_finite_differences():
    model, p, x, y = _tiny_mlp()
    _check_grads_fd(model, p, {}, x, y)


def test_zero_head_gives_log_classes_and_first_k_indices():
    # joint pin of scoring and selection: with a zero classifier every loss is ln C, so the k
    # selected samples are the first k by the index tie-break.
    model = oracle.ResNetCifar()
    p, b = synth.resnet_init(1)
    p["fc.weight"][:] = 0
    p["fc.bias"][:] = 0
    x, y = synth.image_pool(1, 8, 10)
    losses = oracle.score_losses(model, p, b, x, y)
    np.testing.assert_allclose(losses, np.log(10.0), rtol=1e-14)
    assert oracle.topk_by_loss(losses.astype(np.float32), 3).tolist() == [0, 1, 2]


def test_scoring_is_chunk_independent_and_matches_train_forward_without_bn():
    model, p, b, x, y = _tiny_resnet()
    a = oracle.score_losses(model, p, b, x, y, chunk=6)
    c = oracle.score_losses(model, p, b, x, y, chunk=1)
    np.testing.assert_allclose(a, c, rtol=1e-13)
    mlp, mp, mx, my = _tiny_mlp()
    np.testing.assert_allclose(oracle.score_losses(mlp, mp, {}, mx, my),
                               oracle.loss_and_grads(mlp, mp, {}, mx, my)[0], rtol=1e-14)


def test_closed_form_step_from_zero_head():
    # softmax classifier starting at zero: p = 1/C, so one step gives
    # W2 = -lr/B * sum_b (1/C - e_y) h_b^T, b2 = -lr/B * sum_b (1/C - e_y), and fc1 does not move.
    model, p, x, y = _tiny_mlp()
    p["fc2.weight"][:] = 0
    p["fc2.bias"][:] = 0
    mom = {k: np.zeros_like(v) for k, v in p.items()}
    sel = np.arange(12)
    new, _, _, sl = oracle.local_step(model, p, {}, mom, x, y, sel, batch=12, tau=1, lr=0.5)
    h = np.maximum(x @ p["fc1.weight"].T + p["fc1.bias"], 0)
    r = 1.0 / 3 - np.eye(3)[y]
    np.testing.assert_allclose(new["fc2.weight"], -0.5 / 12 * r.T @ h, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(new["fc2.bias"], -0.5 / 12 * r.sum(axis=0), rtol=1e-12, atol=1e-15)
    np.testing.assert_array_equal(new["fc1.weight"], p["fc1.weight"])
    np.testing.assert_allclose(sl, np.log(3.0), rtol=1e-14)


def test_sgd_momentum_recurrence_and_weight_decay():
    g = [synth.normal(6, s, 7) for s in range(5)]
    x, buf = synth.normal(6, 99, 7), np.zeros(7)
    x0 = x.copy()
    total = np.zeros(7)
    for j in range(5):
        x, buf = oracle.sgd_update(x, buf, g[j], lr=0.1, momentum=0.9)
        expect = sum(0.9 ** (j - s) * g[s] for s in range(j + 1))
        np.testing.assert_allclose(buf, expect, rtol=1e-13)
        total += expect
    np.testing.assert_allclose(x, x0 - 0.1 * total, rtol=1e-12)
    x1, b1 = oracle.sgd_update(x0, np.zeros(7), g[0], lr=0.1, momentum=0.0, weight_decay=1e-4)
    np.testing.assert_allclose(x1, x0 - 0.1 * (g[0] + 1e-4 * x0), rtol=1e-14)
    np.testing.assert_allclose(b1, g[0] + 1e-4 * x0, rtol=1e-14)


def test_local_step_order_wrap_and_full_batch_special_case():
    model, p, x, y = _tiny_mlp()
    zeros = {k: np.zeros_like(v) for k, v in p.items()}
    sel = np.array([7, 2, 9, 4, 11], dtype=np.int32)
    # lr = 0 freezes the model, so step j must report the scores of sel[(j*B + b) mod k]
    _, _, _, sl = oracle.local_step(model, p, {}, zeros, x, y, sel, batch=3, tau=4, lr=0.0)
    score = oracle.score_losses(model, p, {}, x, y)
    order = sel[(np.arange(12)) % 5].reshape(4, 3)
    np.testing.assert_allclose(sl, score[order], rtol=1e-14)
    # tau = 1, batch = k = N: one full-batch gradient-descent step
    new, _, mom, _ = oracle.local_step(model, p, {}, zeros, x, y, np.arange(12), batch=12, tau=1, lr=0.2)
    _, grads, _ = oracle.loss_and_grads(model, p, {}, x, y)
    for k in p:
        np.testing.assert_allclose(new[k], p[k] - 0.2 * grads[k], rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(mom[k], grads[k], rtol=1e-13, atol=1e-16)


def test_global_update_identity():
    # x_{t+1} = x_t - lr * sum_i w_i sum_j g^i_j for plain SGD (Section 4.4, definition of the global update)
    model, p, x, y = _tiny_mlp()
    zeros = {k: np.zeros_like(v) for k, v in p.items()}
    taus, w = [3, 3, 1], oracle.weights_from_tau([3, 3, 1])
    names = list(p)
    flat = lambda d: np.concatenate([d[k].reshape(-1) for k in names])
    locals_, gsum = [], []
    for i, tau in enumerate(taus):
        sel = (np.arange(4) * 3 + i) % 12
        cur, acc = p, np.zeros(flat(p).size)
        for j in range(tau):
            ids = sel[(j * 2 + np.arange(2)) % 4]
            _, g, _ = oracle.loss_and_grads(model, cur, {}, x[ids], y[ids])
            acc += flat(g)
            cur = {k: cur[k] - 0.1 * g[k] for k in names}
        gsum.append(acc)
        new, _, _, _ = oracle.local_step(model, p, {}, zeros, x, y, sel, batch=2, tau=tau, lr=0.1)
        locals_.append(flat(new))
    agg = oracle.weighted_aggregate(np.stack(locals_), w)
    np.testing.assert_allclose(agg, flat(p) - 0.1 * sum(wi * g for wi, g in zip(w, gsum)), rtol=1e-12, atol=1e-15)


def test_batchnorm_buffers_follow_the_steps():
    model, p, b, x, y = _tiny_resnet()
    mom = {k: np.zeros_like(v) for k, v in p.items()}
    _, nb, _, _ = oracle.local_step(model, p, b, mom, x, y, np.arange(6), batch=3, tau=2, lr=0.0)
    # with lr = 0 the stem statistics are those of the two batches, folded in with momentum 0.1
    from oracle import layers as L
    rm = np.asarray(b["stem.bn.running_mean"], dtype=np.float64)
    for ids in (slice(0, 3), slice(3, 6)):
        y0 = L.conv3x3(x[ids], p["stem.conv.weight"], 1)
        rm = 0.9 * rm + 0.1 * y0.reshape(-1, 2).mean(axis=0)
    np.testing.assert_allclose(nb["stem.bn.running_mean"], rm, rtol=1e-12)


def test_relu_toggle_is_the_other_one_sided_derivative():
    # A unit whose pre-activation is exactly zero: the default takes derivative 0 (the left limit);
    # toggling it gives derivative 1 (the right limit).  One-sided finite differences pin both.
    from oracle import layers as L
    z = np.array([[-1.0, 0.0, 2.0]])
    r = np.array([[0.3, -0.7, 1.1]])
    f = lambda zz: float((L.relu(zz) * r).sum())
    eps = 1e-7
    left = np.array([(f(z) - f(z - eps * np.eye(3)[i])) / eps for i in range(3)])
    right = np.array([(f(z + eps * np.eye(3)[i]) - f(z)) / eps for i in range(3)])
    np.testing.assert_allclose(L.relu_backward(r, L.relu(z))[0], left, atol=1e-6)
    np.testing.assert_allclose(L.relu_backward(r, L.relu(z), toggle=[1])[0], right, atol=1e-6)
    # probe: without toggles it is loss_and_grads; near-zero units are found where they are planted
    model, p, b, x, y = _tiny_resnet()
    probe = oracle.GradientProbe(model, p, b, x, y)
    _, g, _ = oracle.loss_and_grads(model, p, b, x, y)
    for k in g:
        np.testing.assert_array_equal(probe.grads()[k], g[k])
    assert probe.near_zero_units(1e-9) == []
    units = probe.near_zero_units(0.05)
    assert units and all(abs(probe.cache["z"][n].reshape(-1)[i]) <= 0.05 * np.sqrt(np.mean(probe.cache["z"][n] ** 2)) for n, i in units)
    g2 = probe.grads({units[0][0]: [units[0][1]]})
    assert any(np.abs(g2[k] - g[k]).max() > 0 for k in g)
