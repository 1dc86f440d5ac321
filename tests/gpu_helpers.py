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
