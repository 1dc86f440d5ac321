"""Pins of the epoch sampler oracle (Section 4.2): allocation arithmetic against hand-worked values,
set properties, brute force, special cases and the uniformity of the random parts."""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth
from oracle.sampling import allocation, deal, sample_epoch

HERE = os.path.dirname(os.path.abspath(__file__))


def test_allocation_matches_hand_worked_values():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "allocation.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 7
    for N, tf, pf, ts, ps, lam, nf, k, ns in rows:
        assert allocation(int(N), int(tf), int(pf), int(ts), int(ps), float(lam)) == (int(nf), int(k), int(ns))


def test_index_volume_of_the_papers_example():
    # Section 4.2: for N = 100 000 the indices of one epoch take about 390 KB (4-byte indices)
    nf, k, ns = allocation(100000, 32, 8, 1, 2, 0.5)
    assert nf + ns == 100000
    assert round((nf + ns) * 4 / 1024.0) == 391


def _keys(rs, n):
    return rs.random_sample(n).astype(np.float32)


@pytest.mark.parametrize("N,tf,pf,ts,ps,lam", [(50, 4, 3, 1, 2, 0.5), (64, 32, 8, 1, 2, 0.25), (33, 2, 2, 2, 2, 1.0),
                                               (40, 5, 1, 1, 3, 0.01), (17, 1, 4, 1, 1, 0.6)])
def test_set_properties(N, tf, pf, ts, ps, lam):
    rs = np.random.RandomState(N)
    losses = np.abs(rs.standard_normal(N)).astype(np.float32)
    losses[::5] = losses[0]                                   # ties
    r = sample_epoch(losses, _keys(rs, N), _keys(rs, N), tf, pf, ts, ps, lam)
    nf, k, ns = r["n_fast"], r["k"], r["n_slow"]
    assert nf + ns == N and 0 <= k <= nf
    fast, slow = r["fast_ranked"], r["slow_ranked"]
    assert fast.shape == (nf,) and slow.shape == (ns,)
    assert len(set(fast.tolist())) == nf and len(set(slow.tolist())) == ns       # without replacement
    # the high-loss part is the brute-force top-k (sort by loss descending, index ascending)
    brute = sorted(range(N), key=lambda i: (-float(losses[i]), i))[:k]
    assert fast[:k].tolist() == brute
    # every sample outside the fast set has a loss no larger than the k-th, the fill avoids the high-loss part
    if k:
        assert max(losses[fast[k:]], default=-1) <= losses[fast[k - 1]]
    # dealing: round-robin, sizes differ by at most one, concatenation restores the ranking
    for group, ranked, P in ((r["fast"], fast, pf), (r["slow"], slow, ps)):
        sizes = [len(g) for g in group]
        assert max(sizes) - min(sizes) <= 1 and sum(sizes) == len(ranked)
        for p_, g in enumerate(group):
            assert g.tolist() == ranked[p_::P].tolist()


def test_lambda_one_is_pure_top_k_and_tiny_lambda_is_pure_uniform():
    rs = np.random.RandomState(1)
    N = 30
    losses = rs.standard_normal(N).astype(np.float32)
    uf, us = _keys(rs, N), _keys(rs, N)
    r = sample_epoch(losses, uf, us, 3, 2, 1, 2, 1.0)
    assert r["k"] == r["n_fast"]
    assert r["fast_ranked"].tolist() == oracle.topk_by_loss(losses, r["n_fast"]).tolist()
    r0 = sample_epoch(losses, uf, us, 3, 2, 1, 2, 0.01)
    assert r0["k"] == 0
    assert r0["fast_ranked"].tolist() == oracle.topk_by_loss(uf, r0["n_fast"]).tolist()   # largest keys first
    # the slow draw ignores the losses and the fast draw
    r1 = sample_epoch(-losses, _keys(rs, N), us, 3, 2, 1, 2, 0.5)
    assert r1["slow_ranked"].tolist() == r["slow_ranked"].tolist()
    with pytest.raises(ValueError):
        allocation(10, 1, 1, 1, 1, 0.0)


def test_all_key_orders_give_each_subset_equally_often():
    # N = 5, fast gets 4 of them, 2 by loss and 2 drawn from the remaining 3: over all 3! orders of the
    # remaining keys every pair appears equally often (exactly uniform without replacement)
    losses = np.array([5, 4, 3, 2, 1], dtype=np.float32)
    counts = {}
    for perm in itertools.permutations([0.1, 0.2, 0.3]):
        uf = np.array([0.9, 0.8] + list(perm), dtype=np.float32)
        r = sample_epoch(losses, uf, uf, 4, 1, 1, 1, 0.5)
        assert (r["n_fast"], r["k"], r["n_slow"]) == (4, 2, 1)
        assert r["fast_ranked"][:2].tolist() == [0, 1]
        key = tuple(sorted(r["fast_ranked"][2:].tolist()))
        counts[key] = counts.get(key, 0) + 1
    assert counts == {(2, 3): 2, (2, 4): 2, (3, 4): 2}


def test_inclusion_frequencies_are_uniform():
    rs = np.random.RandomState(7)
    N, draws = 40, 3000
    losses = rs.standard_normal(N).astype(np.float32)
    nf, k, ns = allocation(N, 3, 2, 1, 2, 0.5)                 # 30, 15, 10
    high = set(oracle.topk_by_loss(losses, k).tolist())
    fill_hits, slow_hits = np.zeros(N), np.zeros(N)
    for _ in range(draws):
        r = sample_epoch(losses, _keys(rs, N), _keys(rs, N), 3, 2, 1, 2, 0.5)
        fill_hits[r["fast_ranked"][k:]] += 1
        slow_hits[r["slow_ranked"]] += 1
    p_fill = (nf - k) / (N - k)
    for i in range(N):
        if i in high:
            assert fill_hits[i] == 0
        else:
            assert abs(fill_hits[i] / draws - p_fill) < 5 * np.sqrt(p_fill * (1 - p_fill) / draws)
    p_slow = ns / N
    assert np.all(np.abs(slow_hits / draws - p_slow) < 5 * np.sqrt(p_slow * (1 - p_slow) / draws))


def test_appendix_variants_on_a_case_worked_by_hand():
    """Eight samples, tau_F P_F : tau_S P_S = 3 : 1, so N_F = 6 and N_S = 2; lambda = 1/2.  Worked on paper from the
    appendix's description of unified sampling and of handing the high-loss samples to the slow workers."""
    losses = [5, 1, 7, 3, 8, 2, 6, 4]
    u_fast = [.1, .9, .5, .8, .2, .3, .4, .7]
    u_slow = [.6, .5, .4, .3, .2, .9, .1, .8]
    run = lambda **kw: oracle.sample_epoch(losses, u_fast, u_slow, 3, 1, 1, 1, 0.5, **kw)
    # losses 8, 7, 6 sit at 4, 2, 6; of the rest {0, 1, 3, 5, 7} the largest fast keys are .9, .8, .7 at 1, 3, 7
    sep = run()
    assert sep["fast_ranked"].tolist() == [4, 2, 6, 1, 3, 7] and sep["slow_ranked"].tolist() == [5, 7] and sep["k"] == 3
    # unified: the slow workers get what is left, {0, 5}, larger slow key (.9 at 5) first
    uni = run(scheme="unified")
    assert uni["fast_ranked"].tolist() == [4, 2, 6, 1, 3, 7] and uni["slow_ranked"].tolist() == [5, 0]
    # high loss to the slow workers: k = floor(2 / 2) = 1 -> sample 4, then the largest slow key among the rest (.9 at 5);
    # the fast workers draw six by fast key from all eight: .9 .8 .7 .5 .4 .3 at 1 3 7 2 6 5
    hs = run(high_loss_to="slow")
    assert hs["slow_ranked"].tolist() == [4, 5] and hs["fast_ranked"].tolist() == [1, 3, 7, 2, 6, 5] and hs["k"] == 1
    # ... or, unified, from the six that are left: {0, 1, 2, 3, 6, 7} by fast key .9 .8 .7 .5 .4 .1
    hu = run(scheme="unified", high_loss_to="slow")
    assert hu["slow_ranked"].tolist() == [4, 5] and hu["fast_ranked"].tolist() == [1, 3, 7, 2, 6, 0]


@pytest.mark.parametrize("high_loss_to", ["fast", "slow"])
def test_unified_sampling_covers_every_sample_exactly_once(high_loss_to):
    N = 1000
    losses = synth.loss_array("ties16", N)
    uf, us = (synth.rng.uniform01(synth.inputs.BASE_SEED, 600 + g, N).astype(np.float32) for g in (0, 1))
    r = oracle.sample_epoch(losses, uf, us, 32, 8, 4, 2, 0.3, scheme="unified", high_loss_to=high_loss_to)
    both = np.concatenate([r["fast_ranked"], r["slow_ranked"]])
    assert np.array_equal(np.sort(both), np.arange(N))
    # the group that does not sample by loss holds its share in descending order of its own keys
    other, keys = (r["slow_ranked"], us) if high_loss_to == "fast" else (r["fast_ranked"], uf)
    assert np.all(np.diff(np.asarray(keys)[other]) <= 0)
    # the by-loss group is what the separated scheme gives it
    sep = oracle.sample_epoch(losses, uf, us, 32, 8, 4, 2, 0.3, high_loss_to=high_loss_to)
    name = "fast_ranked" if high_loss_to == "fast" else "slow_ranked"
    assert np.array_equal(r[name], sep[name])
