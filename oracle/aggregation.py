"""System-aware model aggregation (Section 4.3, Eq. 4; aggregation step of Algorithm 1)."""
import numpy as np


def weights_from_tau(tau):
    """w_i = tau_i / sum_j tau_j in float64: workers that performed more local steps weigh more."""
    tau = np.asarray(tau, dtype=np.float64)
    if tau.ndim != 1 or tau.size == 0 or np.any(tau < 0) or tau.sum() <= 0:
        raise ValueError("tau must be a non-empty vector of non-negative step counts, not all zero")
    return tau / tau.sum()


def weighted_aggregate(replicas, weights):
    """x_{t+1}[j] = sum_i w_i * x^i[j], accumulated in float64 for i ascending.

    replicas: [P, d] (any float dtype), weights: [P].  Returns float64 [d].
    """
    x = np.asarray(replicas)
    w = np.asarray(weights, dtype=np.float64)
    if x.ndim != 2 or w.shape != (x.shape[0],):
        raise ValueError("replicas [P, d] and weights [P] expected")
    out = np.zeros(x.shape[1], dtype=np.float64)
    for i in range(x.shape[0]):
        out += w[i] * x[i].astype(np.float64)
    return out
