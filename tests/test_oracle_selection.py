"""Pins for the selection oracle: brute-force rank counting, library sort, hand cases."""
import itertools

import numpy as np
import pytest

import oracle
import synth


def _beats(a, ia, b, ib):
    """True if sample (a, ia) ranks strictly before (b, ib): NaN highest, -0 == +0, lower index wins ties."""
    na, nb = a != a, b != b
    if na != nb:
        return na
    if not na and a != b:
        return a > b
    return ia < ib


def _rank_count_topk(losses, k):
    """Independent definition: the rank of a sample is the number of samples that beat it."""
    n = len(losses)
    out = [None] * n
    for i in range(n):
        r = sum(_beats(float(losses[j]), j, float(losses[i]), i) for j in range(n) if j != i)
        out[r] = i
    return out[:k]


def test_exhaustive_length6_over_special_values():
    vals = [np.float32(1.5), np.float32(-0.0), np.float32(0.0), np.float32(np.nan)]
    for combo in itertools.product(range(4), repeat=6):
        arr = np.array([vals[c] for c in combo], dtype=np.float32)
        expect = _rank_count_topk(arr, 6)
        for k in (0, 1, 3, 6):
            assert oracle.topk_by_loss(arr, k).tolist() == expect[:k]


@pytest.mark.parametrize("kind", synth.LOSS_ARRAY_KINDS)
def test_rank_count_on_seeded_arrays(kind):
    arr = synth.loss_array(kind, 257)
    assert oracle.topk_by_loss(arr, 64).tolist() == _rank_count_topk(arr, 64)


def test_values_match_library_sort_on_distinct_losses():
    arr = synth.loss_array("halfnormal", 5000)
    assert np.unique(arr).size == arr.size
    idx = oracle.topk_by_loss(arr, 1250)
    np.testing.assert_array_equal(arr[idx], np.sort(arr)[::-1][:1250])


def test_hand_cases():
    inf = np.inf
    arr = np.array([1.0, np.nan, inf, -inf, 0.0, -0.0, 1.0, np.nan, 2.0], dtype=np.float32)
    # NaNs first (index order), +inf, 2, the two 1.0 by index, the two zeros by index, -inf
    assert oracle.topk_by_loss(arr, 9).tolist() == [1, 7, 2, 8, 0, 6, 4, 5, 3]
    assert oracle.topk_by_loss(arr, 0).tolist() == []
    eq = np.full(100, 2.302585, dtype=np.float32)
    assert oracle.topk_by_loss(eq, 25).tolist() == list(range(25))
    asc = np.arange(10, dtype=np.float32)
    assert oracle.topk_by_loss(asc, 3).tolist() == [9, 8, 7]
    # duplicates straddling the k-th boundary: only the lowest-index copies get in
    dup = np.array([5, 3, 3, 3, 3, 1], dtype=np.float32)
    assert oracle.topk_by_loss(dup, 3).tolist() == [0, 1, 2]
    perm = oracle.topk_by_loss(synth.loss_array("ties16", 300), 300)
    assert sorted(perm.tolist()) == list(range(300))
    assert perm.dtype == np.int32
    with pytest.raises(ValueError):
        oracle.topk_by_loss(asc, 11)
