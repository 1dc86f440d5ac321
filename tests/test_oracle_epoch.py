"""Pins of the epoch-loop oracle (outer loop of Algorithm 1; schedule of Appendix A.1) and of the two ablation switches
(feature-wise evaluation of the appendix): hand-worked schedule and round structure, special cases that reduce to the
already pinned local step / round, and composition over epochs."""
import os

import numpy as np
import pytest

import oracle
import synth
from oracle.sampling import allocation, deal, sample_epoch

HERE = os.path.dirname(os.path.abspath(__file__))
CFG = synth.workload("mlp")


def _golden(kind):
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "epoch_schedule.txt")) if l.strip() and not l.startswith("#")]
    return [r[1:] for r in rows if r[0] == kind]


def test_learning_rate_schedule_matches_the_settings_tables():
    rows = _golden("lr")
    assert len(rows) >= 16
    for lr0, ms, epoch, want in rows:
        got = oracle.multistep_lr(float(lr0), [int(m) for m in ms.split(",")], 0.1, int(epoch))
        assert abs(got - float(want)) <= 1e-12 * float(want), (lr0, ms, epoch)


def test_rounds_per_epoch_match_hand_worked_cases():
    rows = _golden("rounds")
    assert len(rows) >= 4
    for N, B, tf, pf, ts, ps, want in (map(int, r) for r in rows):
        nf, _, ns = allocation(N, tf, pf, ts, ps, 1.0)
        shares = deal(np.arange(nf), pf) + deal(np.arange(ns), ps)
        assert oracle.rounds_per_epoch(shares, [tf] * pf + [ts] * ps, B) == want


def _setup(n):
    m = oracle.MLP()
    p = synth.mlp_init(CFG["id"], hidden=16)
    x, y = synth.image_pool(CFG["id"], n, 10)
    return m, p, x, y


def _zeros(p):
    return {k: np.zeros_like(v, dtype=np.float64) for k, v in p.items()}


def _keys(seed, e, n):
    return np.random.RandomState(seed).random_sample((e, n)).astype(np.float32)


def test_uniform_sampling_ignores_the_losses_and_is_the_limit_of_a_vanishing_high_loss_share():
    rs = np.random.RandomState(3)
    N = 61
    la, lb = rs.random_sample(N).astype(np.float32), rs.random_sample(N).astype(np.float32)
    uf, us = rs.random_sample(N).astype(np.float32), rs.random_sample(N).astype(np.float32)
    for scheme in ("separated", "unified"):
        a = sample_epoch(la, uf, us, 4, 3, 1, 2, 0.5, scheme, "none")
        b = sample_epoch(lb, uf, us, 4, 3, 1, 2, 0.9, scheme, "none")
        tiny = sample_epoch(la, uf, us, 4, 3, 1, 2, 1e-9, scheme, "fast")       # k = floor(1e-9 * N_F) = 0
        for key in ("fast_ranked", "slow_ranked"):
            assert np.array_equal(a[key], b[key]) and np.array_equal(a[key], tiny[key])
        assert a["k"] == 0 and a["n_fast"] + a["n_slow"] == N
        # the fast draw is the N_F largest fast keys (brute force), whatever the losses
        brute = sorted(range(N), key=lambda i: (-float(uf[i]), i))[:a["n_fast"]]
        assert a["fast_ranked"].tolist() == brute
        if scheme == "unified":
            assert sorted(a["fast_ranked"].tolist() + a["slow_ranked"].tolist()) == list(range(N))
        else:
            assert a["slow_ranked"].tolist() == sorted(range(N), key=lambda i: (-float(us[i]), i))[:a["n_slow"]]


def test_uniform_weights_average_plainly_over_the_workers_that_took_part():
    m, p, x, y = _setup(24)
    ia, ib = np.arange(0, 8), np.arange(8, 16)
    pa = oracle.local_step(m, p, {}, _zeros(p), x, y, ia, 4, 1, 0.1, 0.9)[0]
    pb = oracle.local_step(m, p, {}, _zeros(p), x, y, ib, 4, 3, 0.1, 0.9)[0]
    workers = [dict(tau=1, idx=ia, momentum=_zeros(p)), dict(tau=3, idx=ib, momentum=_zeros(p)), dict(tau=0, idx=ia, momentum=_zeros(p))]
    gp = oracle.communication_round(m, p, {}, workers, x, y, 4, 0.1, 0.9, uniform_weights=True)[0]
    gw = oracle.communication_round(m, p, {}, workers, x, y, 4, 0.1, 0.9)[0]
    for k in p:
        np.testing.assert_allclose(gp[k], 0.5 * pa[k] + 0.5 * pb[k], rtol=0, atol=1e-15)       # balanced average of Section 4.3
        np.testing.assert_allclose(gw[k], 0.25 * pa[k] + 0.75 * pb[k], rtol=0, atol=1e-15)     # Eq. (4)
        assert not np.allclose(gp[k], gw[k])


def test_one_worker_one_round_is_a_local_step_on_the_ranked_table():
    N, B, tau = 24, 4, 6
    m, p, x, y = _setup(N)
    table0 = oracle.score_losses(m, p, {}, x, y)
    order = oracle.topk_by_loss(table0.astype(np.float32), N)
    ref_p, _, ref_m, ref_l = oracle.local_step(m, p, {}, _zeros(p), x, y, order, B, tau, 0.1, 0.9, 1e-4)
    gp, _, gm, table, log = oracle.train_epochs(m, p, {}, [_zeros(p)], x, y, table0, _keys(1, 1, N), _keys(2, 1, N), 1, tau, 1, 0, 0, 1.0,
                                                B, 0.1, 0.9, 1e-4)
    assert log == [(0, 0, 0.1, [tau])]
    for k in p:
        assert np.array_equal(gp[k], ref_p[k]) and np.array_equal(gm[0][k], ref_m[k])
    assert np.array_equal(table[order], ref_l.reshape(-1))          # every sample processed once: its loss is recorded


def test_round_structure_and_table_of_a_ragged_epoch():
    # the small hand-worked case of the golden file: N = 22, B = 2, fast 2 x tau 2, slow 1 x tau 1 -> 3 rounds, steps 2, 0, 1 in the last
    N, B = 22, 2
    m, p, x, y = _setup(N)
    table0 = np.full(N, -5.0)
    uf, us = _keys(4, 1, N), _keys(5, 1, N)
    out = oracle.train_epochs(m, p, {}, [_zeros(p) for _ in range(3)], x, y, table0, uf, us, 1, 2, 2, 1, 1, 0.5, B, 0.05, 0.9)
    assert [(e, r, t) for e, r, _, t in out[4]] == [(0, 0, [2, 2, 1]), (0, 1, [2, 2, 1]), (0, 2, [2, 0, 1])]
    alloc = sample_epoch(table0.astype(np.float32), uf[0], us[0], 2, 2, 1, 1, 0.5)
    seen = set(alloc["fast_ranked"].tolist()) | set(alloc["slow_ranked"].tolist())
    touched = set(np.flatnonzero(out[3] != -5.0).tolist())
    assert touched == seen                                          # exactly the allocated samples got a recorded loss
    # the same rounds by hand: hands are consecutive pieces of each worker's share
    shares = list(alloc["fast"]) + list(alloc["slow"])
    gp, gb, gm, table = p, {}, [_zeros(p) for _ in range(3)], table0
    for r in range(3):
        ws = []
        for share, tau, mom in zip(shares, (2, 2, 1), gm):
            hand = share[r * tau * B:(r + 1) * tau * B]
            ws.append(dict(tau=tau if len(hand) else 0, idx=hand, momentum=mom))
        gp, gb, gm, table = oracle.communication_round(m, gp, gb, ws, x, y, B, 0.05, 0.9, loss_table=table)
    for k in p:
        assert np.array_equal(out[0][k], gp[k])
    assert np.array_equal(out[3], table)


def test_epochs_compose_with_the_schedule_and_carry_table_momentum_and_model():
    N, B = 20, 2
    m, p, x, y = _setup(N)
    table0 = oracle.score_losses(m, p, {}, x, y)
    uf, us = _keys(6, 2, N), _keys(7, 2, N)
    args = dict(tau_f=2, P_f=2, tau_s=1, P_s=1, lam=0.5, batch=B, momentum=0.9, weight_decay=1e-4)
    both = oracle.train_epochs(m, p, {}, [_zeros(p) for _ in range(3)], x, y, table0, uf, us, 2, lr0=0.1, milestones=(1,), gamma=0.5, **args)
    first = oracle.train_epochs(m, p, {}, [_zeros(p) for _ in range(3)], x, y, table0, uf[:1], us[:1], 1, lr0=0.1, **args)
    second = oracle.train_epochs(m, first[0], first[1], first[2], x, y, first[3], uf[1:], us[1:], 1, lr0=0.05, **args)
    for k in p:
        assert np.array_equal(both[0][k], second[0][k])
        assert all(np.array_equal(a[k], b[k]) for a, b in zip(both[2], second[2]))
    assert np.array_equal(both[3], second[3])
    assert [l[2] for l in both[4]] == [0.1, 0.1, 0.05, 0.05]
    # the second epoch ranks the losses the first one recorded: its high-loss part is the top of the carried table
    alloc = sample_epoch(first[3].astype(np.float32), uf[1], us[1], 2, 2, 1, 1, 0.5)
    assert alloc["fast_ranked"][:alloc["k"]].tolist() == oracle.topk_by_loss(first[3].astype(np.float32), alloc["k"]).tolist()
    assert not np.array_equal(first[3], table0)
