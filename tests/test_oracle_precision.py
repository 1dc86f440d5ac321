"""Pins of the oracle's reduced-precision storage model (bf16 activations, fp32 master weights)."""
import numpy as np
import pytest

import oracle
import synth
from oracle.precision import round_bf16


def test_round_bf16_hand_cases():
    # spacing of bf16 at 1.0 is 2^-7; halfway cases go to the even mantissa
    cases = [(1.0, 1.0), (1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7), (1.0 + 2.0 ** -8, 1.0),
             (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6), (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7),
             (-1.0 - 2.0 ** -8, -1.0), (0.0, 0.0), (226.3 * 2.0 ** 120, 226.0 * 2.0 ** 120), (np.inf, np.inf), (-np.inf, -np.inf),
             (2.0 ** -126, 2.0 ** -126), (2.0 ** -133, 2.0 ** -133), (2.0 ** -134, 0.0)]
    for v, want in cases:
        got = float(round_bf16(np.array([v]))[0])
        assert got == want, (v, got, want)
    assert np.isnan(round_bf16(np.array([np.nan]))[0])
    # largest finite float32 rounds up to infinity
    assert np.isinf(round_bf16(np.array([3.4028234e38]))[0])


def test_round_bf16_matches_library_conversion():
    torch = pytest.importorskip("torch")
    rs = np.random.RandomState(3)
    v = np.concatenate([rs.standard_normal(20000) * 10.0 ** rs.uniform(-30, 30, 20000),
                        (1.0 + np.arange(-300, 300) * 2.0 ** -9)]).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(round_bf16(v), want)
    # idempotent, and every result has a zero low half
    again = round_bf16(want)
    np.testing.assert_array_equal(again, want)
    assert not (want.astype(np.float32).view(np.uint32) & 0xFFFF).any()


def _case():
    widths, blocks, hw, batch = (16, 16, 32), 1, 8, 3
    p, b = synth.resnet_init(1, widths, blocks, 10, perturb_bn=0.2)
    x, y = synth.image_pool(1, batch, 10, hw=hw)
    return widths, blocks, p, b, x, y


def test_identity_storage_is_the_plain_model():
    widths, blocks, p, b, x, y = _case()
    plain = oracle.ResNetCifar(widths, blocks)
    calls = []

    def ident(a):
        calls.append(a.shape)
        return a

    hooked = oracle.ResNetCifar(widths, blocks, storage=ident)
    l0, g0, b0 = oracle.loss_and_grads(plain, p, b, x, y)
    l1, g1, b1 = oracle.loss_and_grads(hooked, p, b, x, y)
    np.testing.assert_array_equal(l0, l1)
    for k in g0:
        np.testing.assert_array_equal(g0[k], g1[k])
    # training pass: image, 7 weights, 7 convolution outputs, 7 activations; backward: 7 dy, 3 block
    # input gradients with their 3 shortcut branches, 3 gradients of the mid-block activation
    assert len(calls) == 1 + 7 + 7 + 7 + 7 + 3 + 3 + 3
    calls.clear()
    oracle.score_losses(hooked, p, b, x, y)
    assert len(calls) == 1 + 7 + 7   # inference: no rounding between convolution and batch norm


def test_storage_points_hold_representable_values():
    widths, blocks, p, b, x, y = _case()
    m = oracle.ResNetCifar(widths, blocks, storage=round_bf16)
    logits, cache, _ = m.forward(p, b, x, train=True)
    for name in ["x", "stem.out", "s1.b0.h1", "s1.b0.out", "s3.b0.out"]:
        np.testing.assert_array_equal(cache[name], round_bf16(cache[name]))
    for name, wq in cache["w"].items():
        np.testing.assert_array_equal(wq, round_bf16(p[name]))
    # parameters themselves are untouched and gradients are not rounded
    assert any((cache["p"][k] != round_bf16(cache["p"][k])).any() for k in cache["w"])
    _, g, _ = oracle.loss_and_grads(m, p, b, x, y)
    assert (g["s2.b0.conv1.weight"] != round_bf16(g["s2.b0.conv1.weight"])).any()
    # close to the full-precision model: bf16 carries 8 significant bits
    l_b = oracle.score_losses(m, p, b, x, y)
    l_f = oracle.score_losses(oracle.ResNetCifar(widths, blocks), p, b, x, y)
    assert 0 < np.abs(l_b - l_f).max() < 0.05
