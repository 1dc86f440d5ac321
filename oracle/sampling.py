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

Variants compared in the appendix (sampling-scheme comparison and its table).  scheme "separated" is the
method above.  scheme "unified": the group that samples by loss goes first and the other group trains on
the remaining data, i.e. on exactly the N - N_biased samples the first group did not take, in the order of
its random keys.  high_loss_to "slow" hands the high-loss samples to the slow workers instead: the slow
allocation is the floor(lambda N_S) highest losses plus a uniform fill from the rest, and the fast workers
draw uniformly (from all N, or from the remainder under "unified").  The unbiased baseline of that table (and the
settings of the feature-wise evaluation that switch the sampling bias off) is uniform sampling for both groups and
needs no loss at all: high_loss_to "none" has no by-loss part (k = 0), the fast workers draw their N_F samples by
their keys and the slow workers theirs, independently ("separated") or from what the fast workers left ("unified").
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


def _by_loss_then_uniform(losses, keys, n, k):
    """n ranked indices: the k highest losses, then the n - k largest keys among the rest."""
    high = topk_by_loss(losses, k)                                   # highest loss first, ties by lower index
    unselected = np.ones(losses.shape[0], dtype=bool)
    unselected[high] = False
    rest = np.flatnonzero(unselected)
    # uniform without replacement from the rest: largest random key first
    fill = rest[topk_by_loss(keys[rest], n - k)] if n > k else np.zeros(0, dtype=np.int64)
    return np.concatenate([high.astype(np.int64), fill.astype(np.int64)])


def sample_epoch(losses, u_fast, u_slow, tau_f, P_f, tau_s, P_s, lam, scheme="separated", high_loss_to="fast"):
    """Returns dict(fast=[P_f index arrays], slow=[P_s index arrays], n_fast, k, n_slow, fast_ranked, slow_ranked);
    k is the size of the by-loss part of the group named by high_loss_to."""
    if scheme not in ("separated", "unified") or high_loss_to not in ("fast", "slow", "none"):
        raise ValueError("unknown sampling variant")
    losses = np.asarray(losses, dtype=np.float32)
    u_fast = np.asarray(u_fast, dtype=np.float32)
    u_slow = np.asarray(u_slow, dtype=np.float32)
    N = losses.shape[0]
    n_fast, k, n_slow = allocation(N, tau_f, P_f, tau_s, P_s, lam)
    if high_loss_to == "slow":
        k = int(math.floor(float(lam) * float(n_slow)))
    if high_loss_to == "none":
        k = 0                                                        # nobody samples by loss; the fast group draws first
    n_biased, u_biased, n_other, u_other = (n_slow, u_slow, n_fast, u_fast) if high_loss_to == "slow" else (n_fast, u_fast, n_slow, u_slow)
    biased = _by_loss_then_uniform(losses, u_biased, n_biased, k)
    if scheme == "separated":
        other = topk_by_loss(u_other, n_other).astype(np.int64)      # from all N, independent of the other group
    else:
        left = np.ones(N, dtype=bool)
        left[biased] = False
        left = np.flatnonzero(left)                                  # what the first group did not take
        other = left[topk_by_loss(u_other[left], n_other)].astype(np.int64)
    fast_ranked, slow_ranked = (other, biased) if high_loss_to == "slow" else (biased, other)
    return dict(fast=deal(fast_ranked, P_f), slow=deal(slow_ranked, P_s), n_fast=n_fast, k=k, n_slow=n_slow,
                fast_ranked=fast_ranked, slow_ranked=slow_ranked)
