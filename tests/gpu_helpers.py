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


def assert_grads_match_up_to_relu_ties(probe, got, tol=1e-4, rel_margin=1e-5, max_units=32, what="gradients",
                                       tensors=None, relus=None):
    """Gradients must match the oracle's per tensor (norm-wise `tol`).

    A ReLU unit whose fp64 pre-activation lies within rel_margin * rms of zero can land on either
    side of the kink in fp32; both one-sided derivatives are valid there.  If the plain comparison
    fails, the oracle's decisions for exactly those units (found from the oracle's own forward pass)
    are inverted one at a time, keeping an inversion when it brings the oracle closer; the result
    must then match at `tol`.  Units outside the margin are never touched.  `tensors` restricts the
    comparison to some gradient tensors and `relus` the search to the ReLUs that can influence them.
    """
    def worst(ref):
        return max(rel_err(got[k], ref[k]) for k in ref if tensors is None or k in tensors)

    ref = probe.grads()
    best = worst(ref)
    if best <= tol:
        return 0
    units = [u for u in probe.near_zero_units(rel_margin) if relus is None or u[0] in relus]
    assert units, (what, "no ReLU unit near zero, yet error", best)
    assert len(units) <= max_units, (what, "too many near-zero units to search", len(units))
    toggles, flipped = {}, 0
    for name, idx in units:
        trial = {k: list(v) for k, v in toggles.items()}
        trial.setdefault(name, []).append(idx)
        e = worst(probe.grads(trial))
        if e < best:
            best, toggles, flipped = e, trial, flipped + 1
        if best <= tol:
            break
    assert best <= tol, (what, best, "after inverting", flipped, "of", len(units), "near-zero ReLU units")
    return flipped
