"""One communication round of Algorithm 1 on one set of workers.

Every worker starts from the global model, performs its tau_i local SGD steps on the samples the sampler assigned
to it (the inner loop of Algorithm 1), the individual losses of the processed samples are recorded in the loss table
(the loss-recording step), and the global model becomes the aggregate sum_i (tau_i / sum_j tau_j) x^i of Eq. (4).

Readings where the paper is silent: a worker keeps its own momentum buffers from round to round (they are an input
and an output here); batch-norm running statistics are aggregated with the same weights as the parameters; a sample
processed more than once in a round keeps the loss recorded last, in the order workers (as listed), steps, positions
in the batch; a worker with tau_i = 0 neither trains nor counts.

uniform_weights=True replaces Eq. (4) by the balanced average x_{t+1} = (1/m) sum_i x^i of Section 4.3 over the m
workers that took part (the settings of the feature-wise evaluation without the aggregation bias).
"""
import numpy as np

from .aggregation import weights_from_tau
from .local_sgd import local_step


def communication_round(model, global_params, global_buffers, workers, x_pool, y_pool, batch, lr, momentum=0.0,
                        weight_decay=0.0, loss_table=None, uniform_weights=False):
    """workers: list of dict(tau=int, idx=int array, momentum=dict of arrays).

    Returns (global_params, global_buffers, [momentum dict per worker], loss_table); inputs are not modified.
    """
    taus = [int(w["tau"]) for w in workers]
    weights = weights_from_tau([1 if t > 0 else 0 for t in taus]) if uniform_weights else weights_from_tau(taus)
    table = None if loss_table is None else np.array(loss_table, dtype=np.float64)
    new_p = {k: np.zeros_like(np.asarray(v, dtype=np.float64)) for k, v in global_params.items()}
    new_b = {k: np.zeros_like(np.asarray(v, dtype=np.float64)) for k, v in global_buffers.items()}
    new_m = []
    for w, tau, weight in zip(workers, taus, weights):
        if tau == 0:
            new_m.append({k: np.asarray(v, dtype=np.float64) for k, v in w["momentum"].items()})
            continue
        idx = np.asarray(w["idx"]).astype(np.int64)
        p, b, m, losses = local_step(model, global_params, global_buffers, w["momentum"], x_pool, y_pool, idx, batch, tau, lr,
                                     momentum, weight_decay)
        new_m.append(m)
        if table is not None:
            for j in range(tau):
                for pos in range(batch):
                    table[idx[(j * batch + pos) % idx.shape[0]]] = losses[j, pos]
        for k in new_p:
            new_p[k] += weight * p[k]
        for k in new_b:
            new_b[k] += weight * b[k]
    return new_p, new_b, new_m, table
