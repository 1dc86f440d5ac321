"""Pins of the communication-round oracle (Algorithm 1, one round; Eq. 4): it is a composition, so it is pinned through
its special cases - one worker is a plain local step, zero learning rate leaves the model alone, two workers give the
weighted mean of two separately computed local steps - and the loss table through a sequence written out by hand."""
import numpy as np

import oracle
import synth

CFG = synth.workload("mlp")


def _setup(n=24):
    m = oracle.MLP()
    p = synth.mlp_init(CFG["id"], hidden=16)
    x, y = synth.image_pool(CFG["id"], n, 10)
    return m, p, x, y


def _zeros(p):
    return {k: np.zeros_like(v, dtype=np.float64) for k, v in p.items()}


def test_one_worker_is_a_local_step():
    m, p, x, y = _setup()
    idx = np.array([3, 7, 1, 9, 20, 11])
    ref_p, _, ref_m, ref_l = oracle.local_step(m, p, {}, _zeros(p), x, y, idx, 4, 3, 0.1, 0.9, 1e-4)
    gp, gb, gm, table = oracle.communication_round(m, p, {}, [dict(tau=3, idx=idx, momentum=_zeros(p))], x, y, 4, 0.1, 0.9, 1e-4,
                                                   loss_table=np.full(24, -1.0))
    assert all(np.array_equal(gp[k], ref_p[k]) and np.array_equal(gm[0][k], ref_m[k]) for k in p) and gb == {}
    # positions walked: step 0 -> 3 7 1 9, step 1 -> 20 11 3 7, step 2 -> 1 9 20 11; each sample keeps its last loss
    expect = np.full(24, -1.0)
    expect[[3, 7]] = ref_l[1, 2:4]
    expect[[1, 9, 20, 11]] = ref_l[2]
    assert np.array_equal(table, expect)


def test_two_workers_give_the_weighted_mean_of_their_local_steps_and_later_workers_overwrite_the_table():
    m, p, x, y = _setup()
    ia, ib = np.array([0, 1, 2, 3, 4, 5, 6, 7]), np.array([5, 6, 7, 8, 9, 10])
    pa, _, ma, la = oracle.local_step(m, p, {}, _zeros(p), x, y, ia, 4, 1, 0.1, 0.9)
    pb, _, mb, lb = oracle.local_step(m, p, {}, _zeros(p), x, y, ib, 4, 3, 0.1, 0.9)
    workers = [dict(tau=1, idx=ia, momentum=_zeros(p)), dict(tau=3, idx=ib, momentum=_zeros(p)), dict(tau=0, idx=ia, momentum=_zeros(p))]
    gp, _, gm, table = oracle.communication_round(m, p, {}, workers, x, y, 4, 0.1, 0.9, loss_table=np.zeros(24))
    for k in p:
        np.testing.assert_allclose(gp[k], 0.25 * pa[k] + 0.75 * pb[k], rtol=0, atol=1e-15)
        assert np.array_equal(gm[0][k], ma[k]) and np.array_equal(gm[1][k], mb[k]) and not gm[2][k].any()
    # worker a: 0 1 2 3; worker b: 5 6 7 8 / 9 10 5 6 / 7 8 9 10 -> 5, 6 from its second step, 7 .. 10 from its third
    expect = np.zeros(24)
    expect[[0, 1, 2, 3]] = la[0]
    expect[[5, 6]] = lb[1, 2:4]
    expect[[7, 8, 9, 10]] = lb[2]
    assert np.array_equal(table, expect)


def test_zero_learning_rate_leaves_the_global_model_alone_and_equal_steps_average_plainly():
    m, p, x, y = _setup()
    workers = [dict(tau=2, idx=np.arange(8) + 8 * i, momentum=_zeros(p)) for i in range(3)]
    gp, _, _, _ = oracle.communication_round(m, p, {}, workers, x, y, 4, 0.0)
    for k in p:
        np.testing.assert_allclose(gp[k], np.asarray(p[k], np.float64), rtol=0, atol=1e-15)
    gp, _, _, _ = oracle.communication_round(m, p, {}, workers, x, y, 4, 0.05)
    singles = [oracle.local_step(m, p, {}, _zeros(p), x, y, w["idx"], 4, 2, 0.05)[0] for w in workers]
    for k in p:
        np.testing.assert_allclose(gp[k], sum(s[k] for s in singles) / 3.0, rtol=0, atol=1e-15)


def test_running_statistics_are_aggregated_with_the_same_weights():
    cfg = synth.workload("resnet20_fp32")
    widths, blocks, hw = (16, 16, 16), 1, 8
    m = oracle.ResNetCifar(widths, blocks)
    p, b = synth.resnet_init(cfg["id"], widths, blocks, 10, perturb_bn=0.1)
    x, y = synth.image_pool(cfg["id"], 16, 10, hw=hw)
    ia, ib = np.arange(0, 8), np.arange(8, 16)
    pa, ba, _, _ = oracle.local_step(m, p, b, _zeros(p), x, y, ia, 4, 2, 0.05, 0.9)
    pb, bb, _, _ = oracle.local_step(m, p, b, _zeros(p), x, y, ib, 4, 1, 0.05, 0.9)
    workers = [dict(tau=2, idx=ia, momentum=_zeros(p)), dict(tau=1, idx=ib, momentum=_zeros(p))]
    gp, gb, _, _ = oracle.communication_round(m, p, b, workers, x, y, 4, 0.05, 0.9)
    for k in b:
        np.testing.assert_allclose(gb[k], (2.0 * ba[k] + 1.0 * bb[k]) / 3.0, rtol=0, atol=1e-14)
        assert not np.allclose(ba[k], bb[k])          # the two workers really saw different batches
    for k in p:
        np.testing.assert_allclose(gp[k], (2.0 * pa[k] + 1.0 * pb[k]) / 3.0, rtol=0, atol=1e-14)
