"""GPU parity of sample_epoch against the oracle (bit-exact index lists), and host helpers."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    yield torch, bls, ctx
    ctx.close()


def _keys(seed, stream, n):
    return synth.rng.uniform01(seed, stream, n).astype(np.float32)


def _run(env, losses, uf, us, tf, pf, ts, ps, lam):
    torch, bls, ctx = env
    N = losses.shape[0]
    nf, k, ns = bls.epoch_allocation(N, tf, pf, ts, ps, lam)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    fast = torch.full((max(nf, 1),), -7, dtype=torch.int32, device="cuda")
    slow = torch.full((max(ns, 1),), -7, dtype=torch.int32, device="cuda")
    bls.sample_epoch(ctx, dev(losses), dev(uf), dev(us), tf, pf, ts, ps, lam, fast, slow)
    ctx.synchronize()
    return nf, k, ns, fast.cpu().numpy()[:nf], slow.cpu().numpy()[:ns]


def _check(env, losses, uf, us, tf, pf, ts, ps, lam):
    torch, bls, ctx = env
    nf, k, ns, fast, slow = _run(env, losses, uf, us, tf, pf, ts, ps, lam)
    ref = oracle.sample_epoch(losses, uf, us, tf, pf, ts, ps, lam)
    assert (nf, k, ns) == (ref["n_fast"], ref["k"], ref["n_slow"])
    for got, group, n, P in ((fast, ref["fast"], nf, pf), (slow, ref["slow"], ns, ps)):
        for p in range(P if n else 0):
            off, cnt = bls.worker_share(n, P, p)
            np.testing.assert_array_equal(got[off:off + cnt], group[p].astype(np.int32))


@pytest.mark.parametrize("N,tf,pf,ts,ps,lam", [
    (1, 1, 1, 1, 1, 1.0), (2, 1, 1, 1, 1, 0.5), (50, 4, 3, 1, 2, 0.5), (257, 32, 8, 1, 2, 0.25), (4096, 32, 8, 4, 2, 0.5),
    (5000, 3, 7, 2, 5, 1.0), (5000, 3, 7, 2, 5, 0.001), (16385, 32, 8, 16, 2, 0.3), (100000, 32, 8, 1, 2, 0.5),
    (40000, 2, 2, 0, 0, 0.5), (70001, 1, 1, 5, 3, 0.9),
])
def test_matches_the_oracle(env, N, tf, pf, ts, ps, lam):
    seed = synth.inputs.BASE_SEED + N
    for kind in ("halfnormal", "ties16"):
        losses = synth.loss_array(kind, N, seed=seed)
        _check(env, losses, _keys(seed, 11, N), _keys(seed, 12, N), tf, pf, ts, ps, lam)


def test_special_losses_and_tied_keys(env):
    N = 20000
    losses = synth.loss_array("specials", N)
    uf = np.round(_keys(5, 1, N) * 8).astype(np.float32) / 8          # nine distinct key values: heavy ties
    us = np.zeros(N, dtype=np.float32)                                 # all equal: index order decides
    _check(env, losses, uf, us, 32, 8, 1, 2, 0.5)
    _check(env, synth.loss_array("equal", N), uf, us, 4, 4, 4, 4, 0.75)


def test_paper_sized_pool_properties(env):
    torch, bls, ctx = env
    N, tf, pf, ts, ps, lam = 50000, 32, 8, 1, 2, 0.5
    losses = synth.loss_array("halfnormal", N)
    nf, k, ns, fast, slow = _run(env, losses, _keys(9, 1, N), _keys(9, 2, N), tf, pf, ts, ps, lam)
    assert (nf, k, ns) == (49612, 24806, 388)
    assert len(np.unique(fast)) == nf and len(np.unique(slow)) == ns
    assert fast.min() >= 0 and fast.max() < N and slow.min() >= 0 and slow.max() < N
    # undo the dealing: rank r sits at position r // P of worker r % P
    ranked = np.empty(nf, dtype=np.int64)
    for p in range(pf):
        off, cnt = bls.worker_share(nf, pf, p)
        ranked[p::pf] = fast[off:off + cnt]
    thr = np.sort(losses)[::-1][k - 1]
    assert losses[ranked[:k]].min() >= thr and np.all(np.diff(losses[ranked[:k]]) <= 0)
    assert losses[ranked[k:]].max() <= thr


def test_errors(env):
    torch, bls, ctx = env
    z = torch.zeros(8, device="cuda")
    out = torch.zeros(8, dtype=torch.int32, device="cuda")
    for args in [(0, 1, 1, 1, 0.5), (1, 0, 1, 1, 0.5), (1, 1, 1, 1, 0.0), (1, 1, 1, 1, 1.5), (1, 1, -1, 1, 0.5), (1, 2000, 1, 1, 0.5)]:
        with pytest.raises(bls.BlsError):
            bls.sample_epoch(ctx, z, z, z, args[0], args[1], args[2], args[3], args[4], out, out)
    with pytest.raises(bls.BlsError):
        bls.sample_epoch(ctx, z, z, z, 1, 1, 1, 1, 0.5, None, out)


# ---- the appendix's sampling variants ---------------------------------------------------------------------------------

def _check_variant(env, losses, uf, us, tf, pf, ts, ps, lam, scheme, to):
    torch, bls, ctx = env
    N = losses.shape[0]
    nf, _, ns = bls.epoch_allocation(N, tf, pf, ts, ps, lam)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    fast = torch.full((max(nf, 1),), -7, dtype=torch.int32, device="cuda")
    slow = torch.full((max(ns, 1),), -7, dtype=torch.int32, device="cuda")
    bls.sample_epoch(ctx, dev(losses), dev(uf), dev(us), tf, pf, ts, ps, lam, fast, slow, scheme=scheme, high_loss_to=to)
    ctx.synchronize()
    ref = oracle.sample_epoch(losses, uf, us, tf, pf, ts, ps, lam, scheme=scheme, high_loss_to=to)
    assert (nf, ns) == (ref["n_fast"], ref["n_slow"])
    for got, group, n, P in ((fast.cpu().numpy()[:nf], ref["fast"], nf, pf), (slow.cpu().numpy()[:ns], ref["slow"], ns, ps)):
        for p in range(P if n else 0):
            off, cnt = bls.worker_share(n, P, p)
            np.testing.assert_array_equal(got[off:off + cnt], group[p].astype(np.int32))
    return fast.cpu().numpy()[:nf], slow.cpu().numpy()[:ns]


@pytest.mark.parametrize("scheme,to", [("separated", "fast"), ("unified", "fast"), ("separated", "slow"), ("unified", "slow"),
                                       ("separated", "none"), ("unified", "none")])
@pytest.mark.parametrize("N,tf,pf,ts,ps,lam", [
    (8, 3, 1, 1, 1, 0.5), (257, 32, 8, 1, 2, 0.25), (5000, 3, 7, 2, 5, 1.0), (5000, 3, 7, 2, 5, 0.001), (16385, 32, 8, 16, 2, 0.3),
    (50000, 32, 8, 1, 2, 0.5), (40000, 2, 2, 0, 0, 0.5),
])
def test_variants_match_the_oracle(env, scheme, to, N, tf, pf, ts, ps, lam):
    seed = synth.inputs.BASE_SEED + 3 * N
    for kind in ("halfnormal", "ties16"):
        losses = synth.loss_array(kind, N, seed=seed)
        fast, slow = _check_variant(env, losses, _keys(seed, 21, N), _keys(seed, 22, N), tf, pf, ts, ps, lam, scheme, to)
        if scheme == "unified":
            assert np.array_equal(np.sort(np.concatenate([fast, slow])), np.arange(N))   # every sample exactly once


def test_variants_with_special_losses_tied_keys_and_bad_arguments(env):
    torch, bls, ctx = env
    N = 20000
    losses = synth.loss_array("specials", N)
    uf = np.round(_keys(5, 1, N) * 8).astype(np.float32) / 8
    us = np.zeros(N, dtype=np.float32)
    for scheme in ("separated", "unified"):
        for to in ("fast", "slow", "none"):
            _check_variant(env, losses, uf, us, 32, 8, 4, 2, 0.5, scheme, to)
    # a key of -inf (outside the contract) still never lets a struck sample be drawn twice
    bad = _keys(6, 1, N).copy()
    bad[::3] = -np.inf
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    nf, _, ns = bls.epoch_allocation(N, 32, 8, 4, 2, 0.5)
    fast, slow = torch.empty(nf, dtype=torch.int32, device="cuda"), torch.empty(ns, dtype=torch.int32, device="cuda")
    bls.sample_epoch(ctx, dev(losses), dev(bad), dev(bad), 32, 8, 4, 2, 0.5, fast, slow, scheme="unified", high_loss_to="fast")
    ctx.synchronize()
    assert np.array_equal(np.sort(np.concatenate([fast.cpu().numpy(), slow.cpu().numpy()])), np.arange(N))
    z = torch.zeros(4, dtype=torch.float32, device="cuda")
    o = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(bls.BlsError):
        ctx.check(bls.binding.lib.sample_epoch_variant(ctx.handle, z.data_ptr(), z.data_ptr(), z.data_ptr(), 4, 1, 1, 1, 1, 0.5, 2, 0,
                                                       o.data_ptr(), o.data_ptr()))          # an unknown scheme is rejected
