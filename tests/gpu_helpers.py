"""Shared plumbing of the GPU parity tests: move seeded inputs to the device, call the C ABI
through the binding, bring results back as float64 dicts keyed like the oracle's."""
import numpy as np


class Harness:
    def __init__(self, torch, bls, ctx, model, oracle_model):
        self.torch, self.bls, self.ctx, self.model, self.oracle_model = torch, bls, ctx, model, oracle_model

    def dev(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def score(self, params, buffers, x, y):
        t = self.torch
        p = self.dev(self.model.pack(params))
        b = self.dev(self.model.pack(buffers, buffers=True)) if self.model.num_buffers else None
        out = t.full((max(x.shape[0], 1),), -1.0, dtype=t.float32, device="cuda")
        self.bls.score_losses(self.ctx, self.model, p, b, self.dev(x), self.dev(y), out)
        self.ctx.synchronize()
        return out.cpu().numpy()[:x.shape[0]].astype(np.float64)

    def local_step(self, params, buffers, momentum, x, y, sel, batch, tau, lr, mu=0.0, wd=0.0):
        """Returns (params, buffers, momentum, step_losses) as float64 dicts / array."""
        t = self.torch
        p = self.dev(self.model.pack(params))
        b = self.dev(self.model.pack(buffers, buffers=True)) if self.model.num_buffers else None
        mo = self.dev(self.model.pack(momentum))
        sl = t.full((max(tau * batch, 1),), -1.0, dtype=t.float32, device="cuda")
        self.bls.local_step(self.ctx, self.model, p, b, mo, self.dev(x), self.dev(y), self.dev(np.asarray(sel, np.int32)),
                            batch, tau, lr, mu, wd, sl)
        self.ctx.synchronize()
        f64 = lambda d: {k: v.astype(np.float64) for k, v in d.items()}
        return (f64(self.model.unpack(p.cpu().numpy())),
                f64(self.model.unpack(b.cpu().numpy(), buffers=True)) if b is not None else {},
                f64(self.model.unpack(mo.cpu().numpy())), sl.cpu().numpy()[:tau * batch].astype(np.float64).reshape(tau, batch))


def rel_err(got, ref):
    """Norm-wise relative error of one tensor."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))


def assert_losses_close(got, ref, rtol=1e-4, atol=1e-6):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    bad = np.abs(got - ref) > rtol * np.abs(ref) + atol
    assert not bad.any(), (int(bad.sum()), float(np.max(np.abs(got - ref) / (np.abs(ref) + atol))))


def assert_tensors_close(got, ref, tol=1e-4, what=""):
    worst = {}
    for k in ref:
        e = rel_err(got[k], ref[k])
        if e > tol:
            worst[k] = e
    assert not worst, (what, worst)


def assert_grads_match_up_to_relu_ties(probe, got, tol=1e-4, margins=(3e-6, 1e-5), max_units=256, what="gradients"):
    """Gradients must match the oracle's per tensor (norm-wise `tol`), up to the decisions of ReLU units at the kink.

    A ReLU unit whose fp64 pre-activation lies within a few 1e-6 of the layer's rms of zero can land on either side of the
    kink in fp32; both one-sided derivatives are valid there, so the set of correct results is the oracle's gradient with
    any subset of those units' decisions inverted.  Membership is decided without a search: the backward pass is linear in
    the decision of one unit (and additive over units up to second-order terms far below `tol`), so the difference between
    the kernels' gradient and the oracle's is fitted, by least squares over all tensors (each scaled by its norm), with the
    per-unit effects  grads(unit inverted) - grads()  of exactly the near-zero units, found from the oracle's own forward
    pass.  Units whose coefficient rounds to one are inverted in a real backward pass of the oracle, and that result must
    match at `tol`.  Units outside the margin are never touched.  Returns the number of inverted units.
    """
    ref = probe.grads()
    names = list(ref)
    worst = lambda r: max(rel_err(got[k], r[k]) for k in names)
    if worst(ref) <= tol:
        return 0
    from concurrent.futures import ThreadPoolExecutor
    scale = {k: 1.0 / max(float(np.linalg.norm(ref[k])), 1e-30) for k in names}
    vec = lambda g: np.concatenate([(np.asarray(g[k], np.float64) * scale[k]).reshape(-1) for k in names])
    v0 = vec(ref)
    resid = vec(got) - v0
    effects, best = {}, worst(ref)
    for margin in margins:
        units = probe.near_zero_units(margin)
        assert len(units) <= max_units and len(units) * v0.size <= 4e8, (what, "too many near-zero units", len(units))
        todo = [u for u in units if u not in effects]
        with ThreadPoolExecutor(max_workers=4) as pool:
            for u, e in zip(todo, pool.map(lambda u: (vec(probe.grads({u[0]: [u[1]]})) - v0).astype(np.float32), todo)):
                effects[u] = e
        if not units:
            continue
        E = np.stack([effects[u] for u in units]).astype(np.float64)
        coef, *_ = np.linalg.lstsq(E.T, resid, rcond=None)
        toggles = {}
        for (name, idx), c in zip(units, coef):
            if c > 0.5:
                toggles.setdefault(name, []).append(idx)
        n_inv = sum(len(v) for v in toggles.values())
        best = min(best, worst(probe.grads(toggles))) if toggles else best
        if best <= tol:
            return n_inv
    raise AssertionError((what, "worst tensor error", best, "after fitting the near-zero ReLU units within", margins))
