"""Pins of the oracle's row reduce (A1): top-k under (logit desc, id asc) and row log-sum-exp.

Pinned against library routines and closed forms, never against the oracle's own formula:
numpy lexsort (full stable sort), first-occurrence argmax, scipy float64 logsumexp,
lse of a constant row = c + log V.
"""
import numpy as np
import pytest
from scipy.special import logsumexp

import dt_synth
from oracle import ref


def lexsort_topk(x, k):
    order = np.lexsort((np.arange(len(x)), -x.astype(np.float64)))
    return order[:k]


@pytest.mark.parametrize("V,k", [(8, 3), (1000, 10), (4097, 32), (70000, 12)])
def test_topk_matches_full_sort_f32(V, k):
    rng = np.random.default_rng(V + k)
    x = (rng.standard_normal((5, V)) * 2).astype(np.float32)
    val, idx, lse = ref.topk_rows(x, k)
    for r in range(5):
        want = lexsort_topk(x[r], k)
        assert np.array_equal(idx[r], want)
        assert np.array_equal(val[r], x[r][want])
        assert abs(lse[r] - logsumexp(x[r].astype(np.float64))) < 1e-6 * max(1, abs(lse[r]))


def test_topk_bf16_many_ties_lowest_id_first():
    rng = np.random.default_rng(7)
    x = dt_synth.f32_to_bf16_bits((rng.standard_normal((4, 50000)) * 3).astype(np.float32))
    xf = dt_synth.bf16_bits_to_f32(x)
    k = 32
    val, idx, lse = ref.topk_rows(x, k)
    ties = 0
    for r in range(4):
        want = lexsort_topk(xf[r], k)
        assert np.array_equal(idx[r], want)
        ties += int(np.sum(np.diff(val[r]) == 0))
        # equal values must appear in ascending id order
        for a in range(k - 1):
            if val[r, a] == val[r, a + 1]:
                assert idx[r, a] < idx[r, a + 1]
        assert abs(lse[r] - logsumexp(xf[r].astype(np.float64))) < 2e-6 * abs(lse[r])
    assert ties > 0, "the bf16 case is meant to exercise ties"


def test_topk_duplicates_and_all_equal():
    x = np.zeros((1, 100), np.float32)
    val, idx, lse = ref.topk_rows(x, 7)
    assert np.array_equal(idx[0], np.arange(7))
    assert abs(lse[0] - np.log(100.0)) < 1e-6
    x = np.full((1, 64), 2.5, np.float32)
    x[0, [5, 9, 40]] = 3.0
    val, idx, lse = ref.topk_rows(x, 5)
    assert idx[0].tolist() == [5, 9, 40, 0, 1]


def test_k1_is_first_occurrence_argmax_and_kV_is_full_sort():
    rng = np.random.default_rng(3)
    x = rng.integers(-3, 4, size=(6, 40)).astype(np.float32)  # many duplicates
    val, idx, _ = ref.topk_rows(x, 1)
    assert np.array_equal(idx[:, 0], np.argmax(x, axis=1))   # numpy argmax = first occurrence
    val, idx, _ = ref.topk_rows(x, 40)
    for r in range(6):
        assert np.array_equal(idx[r], lexsort_topk(x[r], 40))


def test_minus_inf_entries_are_not_viable():
    x = np.full((2, 16), -np.inf, np.float32)
    x[0, [3, 11]] = [1.0, 2.0]
    val, idx, lse = ref.topk_rows(x, 4)
    assert idx[0].tolist() == [11, 3, -1, -1]
    assert val[0, 0] == 2.0 and val[0, 1] == 1.0 and np.isneginf(val[0, 2:]).all()
    assert abs(lse[0] - np.log(np.exp(1.0) + np.exp(2.0))) < 1e-6
    assert idx[1].tolist() == [-1] * 4 and np.isneginf(lse[1])


def test_lse_closed_forms():
    for c, V in [(0.0, 10), (-7.25, 1000), (30.0, 128256)]:
        x = np.full((1, V), c, np.float32)
        _, _, lse = ref.topk_rows(x, 1)
        assert abs(lse[0] - (c + np.log(V))) < 4e-6 * max(1.0, abs(c + np.log(V)))
    x = np.full((1, 1000), -50.0, np.float32)
    x[0, 17] = 40.0                                         # one-hot dominant: lse -> max
    _, idx, lse = ref.topk_rows(x, 1)
    assert idx[0, 0] == 17 and lse[0] == np.float32(40.0)
