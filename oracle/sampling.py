"""Epoch sampler of the system-aware biased local SGD framework (Section 4.2; the sampling steps
at the top of every epoch in Algorithm 1).

Fast workers: of N samples they are allocated N_F = N * tau_F P_F / (tau_F P_F + tau_S P_S).  The
lambda * N_F samples with the highest loss come first (deterministic top-k); the remaining
(1 - lambda) * N_F are drawn uniformly without replacement from the samples not yet selected; the
N_F samples are then dealt evenly to the P_F fast workers.  Slow workers: N_S samples drawn uniformly
without replacement from all N samples, independently of the fast workers' draw (so the two groups
may overlap), dealt evenly to the P_S slow workers.

Readings where the paper is silent: N_F = floor of the expression above (exact integer arithmetic),
k = floor(lambda * N_F) in double precision, N_S = N - N_F (the epoch covers N samples); "evenly"
= round-robin by rank, worker p receives ranks p, p + P, p + 2P, ...; uniform sampling without
replacement of m items = the m items with the largest random key, equal keys by lower index, where
the keys (one float per sample and per group) are an input, so that both implementations consume the
same random numbers.
"""
import math

import numpy as np

from .selection import topk_by_loss


def allocation(N, tau_f, P_f, tau_s, P_s, lam):
    """(N_F, k, N_S): fast allocation, its high-loss part, slow allocation."""
    if not (0.0 < lam <= 1.0):
        raise ValueError("lambda must be in (0, 1]")
    n_fast = (int(N) * int(tau_f) * int(P_f)) // (int(tau_f) * int(P_f) + int(tau_s) * int(P_s))
    k = int(math.floor(float(lam) * float(n_fast)))
    return n_fast, k, int(N) - n_fast


def deal(ranked, P):
    """Round-robin by rank: list of P arrays, worker p gets ranked[p], ranked[p + P], ..."""
    return [np.asarray(ranked[p::P]) for p in range(P)]


def sample_epoch(losses, u_fast, u_slow, tau_f, P_f, tau_s, P_s, lam):
    """Returns dict(fast=[P_f index arrays], slow=[P_s index arrays], n_fast, k, n_slow, fast_ranked, slow_ranked)."""
    losses = np.asarray(losses, dtype=np.float32)
    u_fast = np.asarray(u_fast, dtype=np.float32)
    u_slow = np.asarray(u_slow, dtype=np.float32)
    N = losses.shape[0]
    n_fast, k, n_slow = allocation(N, tau_f, P_f, tau_s, P_s, lam)
    high = topk_by_loss(losses, k)                                   # highest loss first, ties by lower index
    unselected = np.ones(N, dtype=bool)
    unselected[high] = False
    rest = np.flatnonzero(unselected)
    # uniform without replacement from the rest: largest random key first
    fill = rest[topk_by_loss(u_fast[rest], n_fast - k)] if n_fast > k else np.zeros(0, dtype=np.int64)
    fast_ranked = np.concatenate([high.astype(np.int64), fill.astype(np.int64)])
    slow_ranked = topk_by_loss(u_slow, n_slow).astype(np.int64)
    return dict(fast=deal(fast_ranked, P_f), slow=deal(slow_ranked, P_s), n_fast=n_fast, k=k, n_slow=n_slow,
                fast_ranked=fast_ranked, slow_ranked=slow_ranked)
