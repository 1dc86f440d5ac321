"""Deterministic loss-based top-k selection (Section 4.2; first sampling step of Algorithm 1).

The fast workers receive the samples "with the highest loss values"; the selection is
deterministic.  The paper leaves ties and non-finite values open.  Reading used here:
a total order in which every NaN ranks above +inf (an unscorable sample counts as hardest),
-0.0 equals +0.0, and equal keys are ordered by ascending sample index.  The result lists the
k selected indices in rank order (largest loss first).
"""
import numpy as np


def total_order_key(losses):
    """(is_nan, value) columns; rank is descending in is_nan, then descending in value."""
    v = np.asarray(losses, dtype=np.float32).astype(np.float64)
    nan = np.isnan(v)
    v = np.where(nan, 0.0, v)
    v = v + 0.0          # -0.0 + 0.0 == +0.0
    return nan, v


def topk_by_loss(losses, k):
    """Indices (int32 [k]) of the k largest losses by a full stable sort of all N keys."""
    losses = np.asarray(losses, dtype=np.float32)
    n = losses.shape[0]
    if not 0 <= k <= n:
        raise ValueError("k must satisfy 0 <= k <= N")
    nan, v = total_order_key(losses)
    idx = np.arange(n)
    # lexsort: last key is the primary one.  NaN first, then larger value, then smaller index.
    order = np.lexsort((idx, -v, ~nan))
    return order[:k].astype(np.int32)
