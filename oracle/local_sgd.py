"""The fast-process local step: score a pool, and run tau local mini-batch SGD updates.

Scoring gives every candidate its current loss value (what the sampler of Section 4.2 ranks);
batch-norm layers use their running statistics there, so a sample's score does not depend on
which other samples are scored with it.  The local step is the inner loop of Algorithm 1 for a
fast worker: tau mini-batch SGD updates (Section 2) on its assigned samples, recording the
individual losses of the processed samples.  Reading for what the paper leaves open: batches
walk the selected list in order and wrap around cyclically, the batch loss is the mean of the
per-sample losses, and batch norm trains with batch statistics.
"""
import numpy as np

from .losses import softmax_cross_entropy
from .optim import sgd_update


def _sample_losses(model, logits, y):
    """(per-sample loss, d loss_b / d logits): models with several predictions per sample average them themselves."""
    if hasattr(model, "sample_losses"):
        return model.sample_losses(logits, y)
    return softmax_cross_entropy(logits, y)


def score_losses(model, params, buffers, x, y, chunk=64):
    """Per-sample loss float64 [N] of every pool item under the current parameters."""
    out = np.empty(x.shape[0], dtype=np.float64)
    for s in range(0, x.shape[0], chunk):
        logits, _, _ = model.forward(params, buffers, x[s:s + chunk], train=False)
        out[s:s + chunk], _ = _sample_losses(model, logits, y[s:s + chunk])
    return out


def loss_and_grads(model, params, buffers, xb, yb):
    """(per-sample losses [B], grads of the mean batch loss, buffers after the forward pass)."""
    logits, cache, new_bufs = model.forward(params, buffers, xb, train=True)
    losses, dlogits = _sample_losses(model, logits, yb)
    grads = model.backward(cache, dlogits / xb.shape[0])
    return losses, grads, new_bufs


class GradientProbe:
    """One training forward pass kept for repeated backward passes with different ReLU decisions.

    near_zero_units(rel) lists the ReLU units whose pre-activation is within rel * rms of zero: there
    an fp32 implementation may land on the other side of the kink, and either one-sided derivative
    is a valid result.  grads(toggles) is the gradient with the listed units' decisions inverted.
    """

    def __init__(self, model, params, buffers, xb, yb):
        logits, self.cache, self.new_buffers = model.forward(params, buffers, xb, train=True)
        self.losses, dlogits = _sample_losses(model, logits, yb)
        self.dlogits = dlogits / xb.shape[0]
        self.model = model

    def grads(self, toggles=None):
        if toggles:
            return self.model.backward(self.cache, self.dlogits, toggles)
        return self.model.backward(self.cache, self.dlogits)

    def near_zero_units(self, rel=1e-5):
        """[(relu name, flat index)] with |z| <= rel * rms(z of that ReLU), closest to zero (relative to the rms) first."""
        out = []
        for name, z in self.cache.get("z", {}).items():
            rms = float(np.sqrt(np.mean(z * z)))
            flat = np.abs(z.reshape(-1))
            for i in np.flatnonzero(flat <= rel * rms):
                out.append((flat[i] / max(rms, 1e-300), name, int(i)))
        out.sort()
        return [(name, i) for _, name, i in out]


def local_step(model, params, buffers, momentum_bufs, x_pool, y_pool, sel, batch, tau,
               lr, momentum=0.0, weight_decay=0.0):
    """tau SGD updates; step j trains on sel[(j*batch + b) mod k], b = 0..batch-1.

    Returns (params, buffers, momentum_bufs, step_losses [tau, batch]); inputs are not modified.
    """
    params = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    buffers = {k: np.asarray(v, dtype=np.float64) for k, v in buffers.items()}
    mom = {k: np.asarray(v, dtype=np.float64) for k, v in momentum_bufs.items()}
    sel = np.asarray(sel).astype(np.int64)
    k = sel.shape[0]
    step_losses = np.zeros((tau, batch), dtype=np.float64)
    for j in range(tau):
        ids = sel[(j * batch + np.arange(batch)) % k]
        losses, grads, buffers = loss_and_grads(model, params, buffers, x_pool[ids], y_pool[ids])
        step_losses[j] = losses
        for name in params:
            params[name], mom[name] = sgd_update(params[name], mom[name], grads[name], lr, momentum, weight_decay)
    return params, buffers, mom, step_losses
