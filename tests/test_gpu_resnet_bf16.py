"""GPU parity of the mixed-precision residual network (bf16 activations, fp32 master weights).

The reference is the float64 oracle evaluated on the bf16 grid (oracle.ResNetCifar(storage=round_bf16)):
the same roundings at the same places, everything between them exact.  Two kinds of checks:

  * Where no rounding decision is a near-tie, the kernels must agree with it as closely as the fp32
    path agrees with the plain oracle.
  * A value that lies within fp32 rounding of the midpoint of two bf16 numbers may legitimately round
    either way, and one such flip changes later roundings in turn.  On deeper nets and larger batches
    this happens somewhere, and the gradient of a randomly initialised network reacts strongly: the
    oracle itself moves by 10-30 % per tensor when its batch-norm parameters are perturbed at the level
    of fp32 rounding.  There the kernels are held to that envelope, measured from the oracle in the
    test, and to tight bounds on what is insensitive (losses, running statistics, classifier gradient).
"""
import numpy as np
import pytest

import oracle
import synth
from gpu_helpers import Harness, assert_losses_close, assert_tensors_close, rel_err

pytestmark = pytest.mark.gpu
CFG = synth.workload("resnet20_bf16")


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    yield torch, bls, ctx
    ctx.close()


def _harness(env, widths=(16, 32, 64), blocks=3, hw=32, classes=10):
    torch, bls, ctx = env
    return Harness(torch, bls, ctx, bls.Model.resnet_cifar(widths, blocks, classes, hw, act_dtype="bf16"),
                   oracle.ResNetCifar(widths, blocks, storage=oracle.round_bf16))


def _zeros(p):
    return {k: np.zeros_like(v) for k, v in p.items()}


def _case(widths, blocks, hw, batch, classes=10):
    p, b = synth.resnet_init(CFG["id"], widths, blocks, classes, perturb_bn=0.2)
    x, y = synth.image_pool(CFG["id"], batch + 5, classes, hw=hw)
    sel = (np.arange(batch) * 3) % (batch + 5)
    return p, b, x, y, sel


def _flip_envelope(model, p, b, xb, yb, ref_grads, eps=1e-5, draws=4, seed=11):
    """Per-tensor change of the oracle's gradients when its batch-norm scales and shifts move by eps relative
    (largest of several draws): how far apart two correct evaluations can be once roundings flip."""
    rs = np.random.RandomState(seed)
    out = {k: 0.0 for k in ref_grads}
    for _ in range(draws):
        p2 = {k: (np.asarray(v, np.float64) * (1.0 + eps * rs.standard_normal(v.shape)) if ".bn" in k else v)
              for k, v in p.items()}
        _, g2, _ = oracle.loss_and_grads(model, p2, b, xb, yb)
        for k in out:
            out[k] = max(out[k], rel_err(g2[k], ref_grads[k]))
    return out


def _inside_envelope(h, p, b, xb, yb, grads, mom, floor=0.02):
    env_err = _flip_envelope(h.oracle_model, p, b, xb, yb, grads)
    return {k: (rel_err(mom[k], grads[k]), env_err[k]) for k in grads
            if rel_err(mom[k], grads[k]) > 2.0 * max(env_err[k], floor)}


SMALL = [((16, 32, 64), 1, 8, 4), ((16, 16, 32), 1, 8, 3), ((64, 64, 64), 1, 8, 2), ((16, 32, 32), 1, 8, 7),
         ((16, 32, 64), 1, 16, 2), ((32, 32, 32), 1, 8, 1)]


def test_small_nets_match_the_bf16_oracle_when_no_rounding_flips(env):
    """Six small nets x four input seeds.  A run without a flipped rounding agrees with the oracle like the
    fp32 path does (1e-4 on every gradient tensor, observed 1e-6); a run with one is 1e-4 .. 1e-1 off and
    must stay inside the envelope.  Every net must have a flip-free seed and so must most runs overall."""
    tight_total, runs = 0, 0
    for widths, blocks, hw, batch in SMALL:
        h = _harness(env, widths, blocks, hw)
        tight_here = 0
        for stream in range(4):
            p, b = synth.resnet_init(CFG["id"], widths, blocks, 10, perturb_bn=0.2)
            x, y = synth.image_pool(CFG["id"], batch + 5, 10, hw=hw, stream=stream)
            sel = (np.arange(batch) * 3) % (batch + 5)
            what = (widths, hw, batch, stream)
            assert_losses_close(h.score(p, b, x, y), oracle.score_losses(h.oracle_model, p, b, x, y), rtol=2e-3)
            losses, grads, new_b = oracle.loss_and_grads(h.oracle_model, p, b, x[sel], y[sel])
            _, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, batch, 1, lr=0.0, mu=0.9)
            worst = max(rel_err(mom[k], grads[k]) for k in grads)
            runs += 1
            if worst <= 1e-4:
                tight_here += 1
                assert_losses_close(sl[0], losses)
                assert_tensors_close(gb, new_b, 1e-5, "running statistics %r" % (what,))
            else:
                assert_losses_close(sl[0], losses, rtol=1e-2)
                assert_tensors_close(gb, new_b, 3e-3, "running statistics %r" % (what,))
                bad = _inside_envelope(h, p, b, x[sel], y[sel], grads, mom)
                assert not bad, (what, bad)
        assert tight_here >= 1, (widths, hw, batch, "no seed without a rounding flip")
        tight_total += tight_here
    assert 2 * tight_total >= runs, (tight_total, runs)


@pytest.mark.parametrize("widths,blocks,hw,batch", [
    ((16, 16, 32), 2, 16, 3),
    ((32, 32, 64), 1, 32, 2),     # stride-2 input gradients, 32-channel stem
    ((16, 64, 64), 1, 16, 5),
    ((16, 32, 64), 3, 32, 16),    # ResNet20
])
def test_larger_nets_stay_inside_the_rounding_flip_envelope(env, widths, blocks, hw, batch):
    h = _harness(env, widths, blocks, hw)
    p, b, x, y, sel = _case(widths, blocks, hw, batch)
    assert_losses_close(h.score(p, b, x, y), oracle.score_losses(h.oracle_model, p, b, x, y), rtol=5e-3)
    losses, grads, new_b = oracle.loss_and_grads(h.oracle_model, p, b, x[sel], y[sel])
    _, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, batch, 1, lr=0.0, mu=0.9)
    assert_losses_close(sl[0], losses, rtol=1e-2)
    assert_tensors_close(gb, new_b, 3e-3, "running statistics")
    floor = 0.02
    bad = _inside_envelope(h, p, b, x[sel], y[sel], grads, mom, floor)
    assert not bad, bad
    # the classifier sees the perturbation only through the pooled features
    assert rel_err(mom["fc.bias"], grads["fc.bias"]) < 2e-2
    # and against the plain float64 model the kernels are no further off than the bf16 oracle is
    plain = oracle.ResNetCifar(widths, blocks)
    _, g64, _ = oracle.loss_and_grads(plain, p, b, x[sel], y[sel])
    for k in grads:
        assert rel_err(mom[k], g64[k]) < 1.5 * rel_err(grads[k], g64[k]) + floor, k


@pytest.mark.parametrize("widths,hw,batch", [
    ((16, 16, 16), 32, 3),    # 16 x 16 channels: six 512-pixel tiles in six pixel groups at 32 x 32, a ragged second tile at 16 x 16
    ((32, 32, 32), 32, 1),    # four channel-block pairs per launch, two tiles
    ((64, 64, 64), 32, 1),    # sixteen pairs
])
def test_pair_weight_gradient_kernel_against_the_oracle(env, widths, hw, batch):
    """Stride-1 layers of at most 64 channels take their weight gradient on the bf16 matrix instruction, one 16 x 16 channel
    block per workgroup (Section 4.1, Eq. (2): the gradient of the local update).  Products of two bf16 numbers are exact in
    fp32, so wherever no rounding to bf16 upstream of a tensor falls on a near-tie the kernels agree with the bf16 oracle as
    tightly as the fp32 path does with the plain one.  The sizes span several tiles, pixel groups and accumulator replicas;
    a run at these sizes usually has a flipped rounding somewhere, and a flip late in the backward pass disturbs only the
    tensors below it, so the criterion is per tensor: over eight seeds every gradient tensor must be tight at least once
    (a kernel that computes something else never is)."""
    h = _harness(env, widths, 1, hw)
    best = {}
    for stream in range(8):
        p, b = synth.resnet_init(CFG["id"], widths, 1, 10, perturb_bn=0.2)
        x, y = synth.image_pool(CFG["id"], batch + 5, 10, hw=hw, stream=stream)
        sel = (np.arange(batch) * 3) % (batch + 5)
        losses, grads, new_b = oracle.loss_and_grads(h.oracle_model, p, b, x[sel], y[sel])
        _, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, batch, 1, lr=0.0, mu=0.9)
        errs = {k: rel_err(mom[k], grads[k]) for k in grads}
        assert max(errs.values()) < 0.6, errs
        if max(errs.values()) <= 1e-4:
            assert_losses_close(sl[0], losses)
        best = {k: min(e, best.get(k, 1.0)) for k, e in errs.items()}
    # the tensors at the very end of the backward pass see every flip above them
    bottom = ("stem.", "s1.b0.conv1.", "s1.b0.bn1.")
    assert not {k: e for k, e in best.items() if e > (2e-3 if k.startswith(bottom) else 1e-4)}, best


def test_pair_weight_gradient_several_tiles_per_workgroup(env):
    """64 -> 64 channels at 8 x 8 maps, 160 images: sixteen channel-block pairs leave sixteen pixel groups for twenty tiles,
    so a workgroup of the kernel walks two tiles and the last groups are ragged.  At this size some bf16 roundings flip, so
    the criterion is the envelope one: no further from the float64 oracle than the bf16 oracle itself is (x 1.5, + 0.03)."""
    widths, hw, batch = (64, 64, 64), 8, 160
    h = _harness(env, widths, 1, hw)
    p, b, x, y, sel = _case(widths, 1, hw, batch)
    losses, grads, new_b = oracle.loss_and_grads(h.oracle_model, p, b, x[sel], y[sel])
    _, gb, mom, sl = h.local_step(p, b, _zeros(p), x, y, sel, batch, 1, lr=0.0, mu=0.9)
    assert_losses_close(sl[0], losses, rtol=2e-2)
    _, g64, _ = oracle.loss_and_grads(oracle.ResNetCifar(widths, 1), p, b, x[sel], y[sel])
    for k in grads:
        assert rel_err(mom[k], g64[k]) < 1.5 * rel_err(grads[k], g64[k]) + 0.03, k


def test_steps_selection_and_determinism_at_the_workload_sizes(env):
    """Pool 4096, k 1024, batch 128, 50 steps: scores against the oracle on a sample of the pool, the
    selection bit for bit from the library's own scores, and the properties of the steps that hold at
    any size."""
    torch, bls, ctx = env
    h = _harness(env)
    N, k, B, tau = CFG["pool"], CFG["k"], CFG["batch"], CFG["tau"]
    p, b = synth.resnet_init(CFG["id"], perturb_bn=0.1)
    x, y = synth.image_pool(CFG["id"], N, CFG["classes"])
    got = h.score(p, b, x, y)
    sample = (np.arange(96) * 41 + 7) % N
    assert_losses_close(got[sample], oracle.score_losses(h.oracle_model, p, b, x[sample], y[sample]), rtol=5e-3)
    assert np.isfinite(got).all()
    dl = torch.from_numpy(got.astype(np.float32)).cuda()
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    bls.topk_by_loss(ctx, dl, k, idx)
    ctx.synchronize()
    sel = idx.cpu().numpy()
    np.testing.assert_array_equal(sel, oracle.topk_by_loss(got.astype(np.float32), k))
    # lr = 0: weights stay, every pass over the selection (k / B = 8 steps) records the same losses for
    # a batch as long as the running statistics do not enter (training mode uses batch statistics)
    p2, b2, m2, sl = h.local_step(p, b, _zeros(p), x, y, sel, B, 2 * (k // B), lr=0.0, mu=0.0)
    np.testing.assert_array_equal(sl[:k // B], sl[k // B:])
    for name in p:
        np.testing.assert_array_equal(p2[name], np.asarray(p[name], np.float64))
    # batch 0 of the steps is scored in training mode: compare with the oracle's training pass
    l0, _, _ = oracle.loss_and_grads(h.oracle_model, p, b, x[sel[:B]], y[sel[:B]])
    assert_losses_close(sl[0], l0, rtol=1e-2)
    # the real settings: finite, repeatable bit for bit, and the loss of the selected samples goes down
    r1 = h.local_step(p, b, _zeros(p), x, y, sel, B, tau, CFG["lr"], CFG["momentum"], CFG["weight_decay"])
    r2 = h.local_step(p, b, _zeros(p), x, y, sel, B, tau, CFG["lr"], CFG["momentum"], CFG["weight_decay"])
    for a_, b_ in zip(r1[:3], r2[:3]):
        for name in a_:
            assert np.isfinite(a_[name]).all(), name
            np.testing.assert_array_equal(a_[name], b_[name])
    np.testing.assert_array_equal(r1[3], r2[3])
    assert r1[3][-8:].mean() < r1[3][:8].mean()


def test_bf16_and_fp32_paths_agree_to_bf16_accuracy(env):
    torch, bls, ctx = env
    p, b = synth.resnet_init(CFG["id"], perturb_bn=0.1)
    x, y = synth.image_pool(CFG["id"], 64, 10)
    hb = _harness(env)
    hf = Harness(torch, bls, ctx, bls.Model.resnet_cifar(), oracle.ResNetCifar())
    sb, sf = hb.score(p, b, x, y), hf.score(p, b, x, y)
    assert 1e-6 < np.abs(sb - sf).max() < 0.05


def test_mlp_rejects_bf16(env):
    torch, bls, ctx = env
    with pytest.raises(bls.BlsError):
        bls.Model(0, act_dtype="bf16")


def test_event_timing_covers_every_dispatch_and_leaves_results_alone(env):
    """The per-class event timing brackets every launch of a step, also the bf16 weight-gradient kernel of the
    64-channel layers, and a timed step gives the bits of an untimed one."""
    torch, bls, ctx = env
    h = _harness(env, widths=(16, 32, 64), blocks=1, hw=16)
    p, b, x, y, sel = _case((16, 32, 64), 1, 16, 8)
    plain = h.local_step(p, b, _zeros(p), x, y, sel, 8, 2, lr=0.05, mu=0.9)
    ctx.profile_begin()
    timed = h.local_step(p, b, _zeros(p), x, y, sel, 8, 2, lr=0.05, mu=0.9)
    prof = ctx.profile_end()
    assert prof["conv_wgrad"][1] > 0 and prof["conv_wgrad"][0] > 0.0 and prof["conv_fwd"][1] > 0
    assert all(ms >= 0.0 for ms, _ in prof.values())
    assert all(np.array_equal(plain[0][k], timed[0][k]) for k in plain[0]) and np.array_equal(plain[3], timed[3])
    torch.cuda.synchronize()   # an error left behind by the timing would surface here
