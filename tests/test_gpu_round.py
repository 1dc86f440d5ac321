"""GPU parity of communication_round (one round of Algorithm 1 on one GPU) against the oracle's round."""
import numpy as np
import pytest

import oracle
import synth
from gpu_helpers import assert_losses_close, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    yield torch, bls, ctx
    ctx.close()


def _zeros(p):
    return {k: np.zeros_like(v, dtype=np.float64) for k, v in p.items()}


def _round(env, model, omodel, p, b, x, y, workers, batch, lr, mu, wd, N, uniform=False):
    """Runs the round on both sides; workers: list of (tau, idx, momentum dict)."""
    torch, bls, ctx = env
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    gp = dev(model.pack(p))
    gb = dev(model.pack(b, buffers=True)) if model.num_buffers else None
    table0 = np.full(N, -3.0, dtype=np.float32)
    table = dev(table0)
    dws = []
    for tau, idx, mom in workers:
        dws.append(dict(tau=tau, idx=dev(np.asarray(idx, np.int32)), params=torch.full_like(gp, 7.0),
                        buffers=torch.full_like(gb, 7.0) if gb is not None else None, momentum=dev(model.pack(mom))))
    bls.communication_round(ctx, model, gp, gb, dws, dev(x), dev(y), batch, lr, mu, wd, table, flags=bls.ROUND_UNIFORM_WEIGHTS if uniform else 0)
    ctx.synchronize()
    ref_p, ref_b, ref_m, ref_t = oracle.communication_round(omodel, p, b, [dict(tau=t, idx=i, momentum=m) for t, i, m in workers], x, y,
                                                            batch, lr, mu, wd, loss_table=table0, uniform_weights=uniform)
    got_p = model.unpack(gp.cpu().numpy())
    got_b = model.unpack(gb.cpu().numpy(), buffers=True) if gb is not None else {}
    got_m = [model.unpack(w["momentum"].cpu().numpy()) for w in dws]
    return got_p, got_b, got_m, table.cpu().numpy(), ref_p, ref_b, ref_m, ref_t, table0


def _compare(p, got_p, got_b, got_m, got_t, ref_p, ref_b, ref_m, ref_t, table0, workers, tol):
    for k in ref_p:   # the change of the global model, up to the fp32 rounding of the parameter itself
        change = np.linalg.norm(ref_p[k] - p[k])
        assert np.linalg.norm(got_p[k] - ref_p[k]) <= tol * change + 4 * 2.0 ** -24 * np.linalg.norm(ref_p[k]), k
    for k in ref_b:
        assert rel_err(got_b[k], ref_b[k]) <= tol, k
    for (tau, _, mom), gm, rm in zip(workers, got_m, ref_m):
        for k in rm:
            if tau == 0:
                assert np.array_equal(gm[k], np.asarray(mom[k], np.float32)), k     # an idle worker's state is not touched
            else:
                assert rel_err(gm[k], rm[k]) <= tol, k
    touched = ref_t != table0.astype(np.float64)
    assert np.array_equal(got_t[~touched], table0[~touched])                        # other entries are left alone
    assert_losses_close(got_t[touched], ref_t[touched], rtol=1e-4)


def test_mlp_round_with_wraparound_overlap_and_an_idle_worker(env):
    torch, bls, ctx = env
    cfg = synth.workload("mlp")
    N = 40
    model, omodel = bls.Model.mlp(hidden=32), oracle.MLP()
    p = synth.mlp_init(cfg["id"], hidden=32)
    x, y = synth.image_pool(cfg["id"], N, 10)
    workers = [(3, np.arange(0, 10), _zeros(p)),                       # 12 positions over 10 samples: two are seen twice
               (1, np.array([8, 9, 20, 21, 22, 23]), _zeros(p)),       # overlaps the first worker: its losses win in the table
               (0, np.arange(30, 34), {k: np.ones_like(v, dtype=np.float64) for k, v in p.items()}),
               (2, np.arange(24, 32), _zeros(p))]
    out = _round(env, model, omodel, p, {}, x, y, workers, 4, 0.05, 0.9, 1e-4, N)
    _compare(p, *out, workers, 1e-4)


@pytest.mark.parametrize("uniform", [False, True])
def test_resnet_round_aggregates_running_statistics_too(env, uniform):
    # uniform: the balanced average of Section 4.3 instead of Eq. (4) (unequal step counts, so the two differ)
    torch, bls, ctx = env
    cfg = synth.workload("resnet20_fp32")
    widths, blocks, hw, N = (16, 16, 32), 1, 8, 24
    model, omodel = bls.Model.resnet_cifar(widths, blocks, 10, hw), oracle.ResNetCifar(widths, blocks)
    p, b = synth.resnet_init(cfg["id"], widths, blocks, 10, perturb_bn=0.1)
    x, y = synth.image_pool(cfg["id"], N, 10, hw=hw)
    workers = [(2, np.arange(0, 8), _zeros(p)), (1, np.arange(8, 16), _zeros(p)), (3, np.arange(12, 24), _zeros(p))]
    out = _round(env, model, omodel, p, b, x, y, workers, 4, 0.05, 0.9, 0.0, N, uniform)
    _compare(p, *out, workers, 2e-3)


def test_rejected_arguments(env):
    torch, bls, ctx = env
    model = bls.Model.mlp(hidden=32)
    gp = torch.zeros(model.num_params, device="cuda")
    x, y = torch.zeros(4, 32, 32, 3, device="cuda"), torch.zeros(4, dtype=torch.int32, device="cuda")
    idx = torch.arange(4, dtype=torch.int32, device="cuda")
    w = dict(tau=1, idx=idx, params=torch.zeros_like(gp), buffers=None, momentum=torch.zeros_like(gp))
    with pytest.raises(bls.BlsError):
        bls.communication_round(ctx, model, gp, None, [dict(w, tau=0)], x, y, 2, 0.1)          # nobody takes a step
    with pytest.raises(bls.BlsError):
        bls.communication_round(ctx, model, gp, None, [dict(w, params=gp)], x, y, 2, 0.1)      # would train in the global vector
    with pytest.raises(bls.BlsError):
        bls.communication_round(ctx, model, gp, None, [w] * 65, x, y, 2, 0.1)                  # more workers than the aggregation takes
    with pytest.raises(bls.BlsError):
        bls.communication_round(ctx, model, gp, None, [w, dict(w)], x, y, 2, 0.1)              # two workers in the same storage
    with pytest.raises(bls.BlsError):
        bls.communication_round(ctx, model, gp, None, [dict(w, momentum=w["params"])], x, y, 2, 0.1)   # momentum inside the replica
    with pytest.raises(bls.BlsError):
        bls.communication_round(ctx, model, gp, None, [w], x, y, 2, 0.1, flags=8)              # unknown flag


def test_workers_side_by_side_give_the_same_bits(env):
    """Three lanes against one: same global model, momenta, running statistics and loss table, bit for bit, twice in a row
    (the second round starts from the first round's aggregate while the lanes are still warm)."""
    torch, bls, ctx = env
    cfg = synth.workload("resnet20_fp32")
    widths, blocks, hw, N = (16, 16, 32), 1, 8, 40
    model = bls.Model.resnet_cifar(widths, blocks, 10, hw)
    p, b = synth.resnet_init(cfg["id"], widths, blocks, 10, perturb_bn=0.1)
    x, y = synth.image_pool(cfg["id"], N, 10, hw=hw)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dx, dy = dev(x), dev(y)
    segments = [np.arange(0, 8), np.arange(6, 16), np.arange(16, 24), np.arange(20, 36), np.arange(30, 40)]
    taus = [2, 1, 3, 2, 1]

    def run(lanes):
        ctx.set_lanes(lanes)
        gp, gb = dev(model.pack(p)), dev(model.pack(b, buffers=True))
        table = torch.full((N,), -3.0, device="cuda")
        ws = [dict(tau=t, idx=dev(s.astype(np.int32)), params=torch.empty_like(gp), buffers=torch.empty_like(gb), momentum=torch.zeros_like(gp))
              for t, s in zip(taus, segments)]
        for _ in range(2):
            bls.communication_round(ctx, model, gp, gb, ws, dx, dy, 4, 0.05, 0.9, 1e-4, table)
        ctx.synchronize()
        torch.cuda.synchronize()
        return [gp.cpu().numpy(), gb.cpu().numpy(), table.cpu().numpy()] + [w["momentum"].cpu().numpy() for w in ws]

    try:
        one, three, five = run(1), run(3), run(5)
    finally:
        ctx.set_lanes(1)
    for a, c, e in zip(one, three, five):
        assert np.array_equal(a, c) and np.array_equal(a, e)
    seen = set()
    for t, seg in zip(taus, segments):
        seen.update(seg[:min(len(seg), 4 * t)].tolist())
    assert np.isfinite(one[0]).all() and (one[2] != -3.0).sum() == len(seen)


@pytest.mark.parametrize("act", ["f32", "bf16"])
def test_workers_inside_one_launch_give_the_same_bits_as_one_after_the_other(env, act):
    """Residual networks run the workers of a round side by side inside the kernels (one launch per layer for all workers
    that still have steps to take; unequal step counts, an idle worker, overlapping samples, selections of different
    lengths): replicas, momenta, running statistics, loss table and aggregate are the same bits as with
    BLS_ROUND_SEQUENTIAL, twice in a row."""
    torch, bls, ctx = env
    cfg = synth.workload("resnet20_fp32")
    widths, blocks, hw, N = (16, 32, 64), 1, 16, 64
    model = bls.Model.resnet_cifar(widths, blocks, 10, hw, act_dtype=act)
    p, b = synth.resnet_init(cfg["id"], widths, blocks, 10, perturb_bn=0.1)
    x, y = synth.image_pool(cfg["id"], N, 10, hw=hw)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dx, dy = dev(x), dev(y)
    segments = [np.arange(0, 12), np.arange(6, 16), np.arange(16, 24), np.arange(3, 9), np.arange(20, 50), np.arange(40, 64)]
    taus = [2, 1, 3, 0, 2, 3]

    def run(flags):
        gp, gb = dev(model.pack(p)), dev(model.pack(b, buffers=True))
        table = torch.full((N,), -3.0, device="cuda")
        ws = [dict(tau=t, idx=dev(s.astype(np.int32)), params=torch.full_like(gp, 5.0), buffers=torch.full_like(gb, 5.0),
                   momentum=torch.full_like(gp, 0.01 * (i + 1))) for i, (t, s) in enumerate(zip(taus, segments))]
        for _ in range(2):
            bls.communication_round(ctx, model, gp, gb, ws, dx, dy, 6, 0.05, 0.9, 1e-4, table, flags=flags)
        ctx.synchronize()
        out = [gp.cpu().numpy(), gb.cpu().numpy(), table.cpu().numpy()]
        for w in ws:
            out += [w["params"].cpu().numpy(), w["buffers"].cpu().numpy(), w["momentum"].cpu().numpy()]
        return out

    side_by_side, in_turn = run(0), run(bls.ROUND_SEQUENTIAL)
    for a, c in zip(side_by_side, in_turn):
        assert np.array_equal(a, c)
    assert np.isfinite(side_by_side[0]).all() and (side_by_side[3 + 3 * 3] == 5.0).all()    # the idle worker's storage is not touched


def test_transformer_round_with_token_sequences(env):
    """The round with the sequence model (int32 token pool, no buffers, bf16 factors): against the oracle's round."""
    torch, bls, ctx = env
    cfg = synth.workload("transformer")
    vocab, L, D, H, F, layers, N = 120, 12, 32, 4, 64, 1, 20
    model = bls.Model.transformer(vocab, L, D, H, F, layers, "bf16")
    omodel = oracle.TransformerLM(vocab, L, D, H, F, layers, operand=oracle.round_bf16)
    p = synth.transformer_init(cfg["id"], vocab, L, D, F, layers, perturb=0.1)
    x, y = synth.token_pool(cfg["id"], N, L, vocab)
    workers = [(2, np.arange(0, 8), _zeros(p)), (1, np.arange(6, 12), _zeros(p)), (2, np.arange(12, 20), _zeros(p))]
    got_p, got_b, got_m, got_t, ref_p, ref_b, ref_m, ref_t, table0 = _round(env, model, omodel, p, {}, x, y, workers, 4, 0.05, 0.9, 0.0, N)
    keep = [k for k in ref_p if not k.endswith("attn.k.bias")]     # zero gradient up to rounding, see the transformer tests
    for k in keep:
        change = np.linalg.norm(ref_p[k] - p[k])
        assert np.linalg.norm(got_p[k] - ref_p[k]) <= 1e-2 * change + 4 * 2.0 ** -24 * np.linalg.norm(ref_p[k]), k
    touched = ref_t != table0.astype(np.float64)
    assert touched.sum() == 18 and np.array_equal(got_t[~touched], table0[~touched])
    assert_losses_close(got_t[touched], ref_t[touched], rtol=1e-3)
