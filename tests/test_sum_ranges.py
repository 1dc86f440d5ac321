"""The fixed-point batch sums of the library have a documented range (include/bls.h, bls_sum_limits).  CPU side: the
limits are what the header states, and the oracle's own forward pass shows that the scaled-input parity case below lies
inside them while the out-of-range case lies outside.  GPU side: inputs thirty times the usual scale still match the
oracle; beyond the range, or with a non-finite input, the results are NaN instead of finite garbage."""
import numpy as np
import pytest

import oracle
import synth
from oracle import layers as L

WIDTHS, BLOCKS, HW, BATCH = (16, 16, 32), 1, 16, 12


def _inputs(scale):
    p, b = synth.resnet_init(1, WIDTHS, BLOCKS, 10, perturb_bn=0.2)
    x, y = synth.image_pool(1, BATCH, 10, hw=HW)
    return p, b, (x * scale).astype(np.float32), y


def _largest_tile_sum_of_squares(p, x):
    """Largest sum of squares of 256 consecutive outputs (pixels x one channel) of the stem convolution: what one
    workgroup adds to a forward statistic."""
    y0 = L.conv3x3(x.astype(np.float64), np.asarray(p["stem.conv.weight"], np.float64), 1)
    flat = (y0 ** 2).reshape(-1, y0.shape[-1])
    tiles = flat[:flat.shape[0] // 256 * 256].reshape(-1, 256, y0.shape[-1]).sum(axis=1)
    return float(tiles.max())


def test_limits_are_the_documented_ones_and_bracket_the_test_cases():
    import paper_2508_08540_amd as bls
    fwd, bwd, wg = bls.sum_limits()
    assert (fwd, bwd, wg) == (2.0 ** 24, 2.0 ** 9, 2.0 ** 13)
    p, b, x30, y = _inputs(30.0)
    assert _largest_tile_sum_of_squares(p, x30) < 0.05 * fwd          # the scaled parity case is well inside the range
    p, b, x255, y = _inputs(1.0)
    raw = np.clip(np.round(60.0 * x255 + 128.0), 0, 255).astype(np.float32)   # 8-bit pixel values
    assert _largest_tile_sum_of_squares(p, raw) < fwd
    p, b, xbig, y = _inputs(3000.0)
    assert _largest_tile_sum_of_squares(p, xbig) > 4.0 * fwd           # the out-of-range case really is out of range


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    yield torch, bls, ctx
    ctx.close()


def _harness(env):
    from gpu_helpers import Harness
    torch, bls, ctx = env
    return Harness(torch, bls, ctx, bls.Model.resnet_cifar(WIDTHS, BLOCKS, 10, HW), oracle.ResNetCifar(WIDTHS, BLOCKS))


def _zeros(p):
    return {k: np.zeros_like(v) for k, v in p.items()}


@pytest.mark.gpu
def test_inputs_thirty_times_larger_still_match_the_oracle(env):
    from gpu_helpers import assert_grads_match_up_to_relu_ties, assert_losses_close, assert_tensors_close
    h = _harness(env)
    p, b, x, y = _inputs(30.0)
    sel = np.arange(BATCH)
    assert_losses_close(h.score(p, b, x, y), oracle.score_losses(h.oracle_model, p, b, x, y))
    probe = oracle.GradientProbe(h.oracle_model, p, b, x, y)
    _, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, BATCH, 1, lr=0.0, mu=0.9)
    assert_losses_close(sl[0], probe.losses)
    assert_grads_match_up_to_relu_ties(probe, mom, 1e-4)
    assert_tensors_close(gb, probe.new_buffers, 1e-5, "running statistics")


@pytest.mark.gpu
@pytest.mark.parametrize("case", ["beyond the range", "a NaN pixel", "an infinite pixel"])
def test_out_of_range_or_non_finite_sums_end_in_nan_not_in_finite_garbage(env, case):
    h = _harness(env)
    p, b, x, y = _inputs(3000.0 if case == "beyond the range" else 1.0)
    if case == "a NaN pixel":
        x[3, 5, 7, 1] = np.nan
    if case == "an infinite pixel":
        x[3, 5, 7, 1] = np.inf
    sel = np.arange(BATCH)
    newp, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, BATCH, 2, lr=0.05, mu=0.9)
    # the step that met the bad sum leaves NaN gradients and parameters behind, and the next step's losses are NaN
    assert all(np.isnan(v).all() for k, v in mom.items() if "conv" in k), {k: float(np.isnan(v).mean()) for k, v in mom.items()}
    assert all(np.isnan(v).all() for k, v in newp.items() if "conv" in k) and np.isnan(newp["fc.weight"]).any()
    assert np.isnan(sl[1]).all()
    # the same model with inputs in range is finite (the scratch carries nothing over)
    p, b, x, y = _inputs(1.0)
    newp, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, BATCH, 2, lr=0.05, mu=0.9)
    assert all(np.isfinite(v).all() for v in newp.values()) and np.isfinite(sl).all()
