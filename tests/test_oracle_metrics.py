"""Pins of the oracle's evaluation metrics (oracle/metrics.py), CPU only: brute force over all
k-subsets for pass@k, the standard library's median, hand-computed speedups and accuracies."""
import itertools
import math
import statistics
from fractions import Fraction

import numpy as np
import pytest

from oracle import metrics as M


@pytest.mark.parametrize("n", [1, 2, 5, 8])
def test_pass_at_k_is_the_fraction_of_subsets_with_a_correct_sample(n):
    for c in range(n + 1):
        samples = [1] * c + [0] * (n - c)
        for k in range(1, n + 1):
            subsets = list(itertools.combinations(range(n), k))
            hits = sum(1 for sub in subsets if any(samples[i] for i in sub))
            assert M.pass_at_k(n, c, k) == Fraction(hits, len(subsets)), (n, c, k)


def test_pass_at_k_special_cases():
    assert M.pass_at_k(10, 0, 3) == 0
    assert M.pass_at_k(10, 10, 3) == 1
    assert M.pass_at_k(10, 3, 1) == Fraction(3, 10)            # k = 1: the plain success rate
    assert M.pass_at_k(10, 8, 3) == 1                          # fewer than k wrong samples: every subset has a hit
    assert M.pass_at_k(4, 1, 2) == Fraction(1, 2)              # by hand: 3 of the 6 pairs hold the correct sample
    with pytest.raises(ValueError):
        M.pass_at_k(3, 1, 4)


def test_median_against_the_standard_library():
    rng = np.random.default_rng(0)
    for n in (1, 2, 3, 4, 7, 10, 101):
        v = rng.random(n).tolist()
        assert M.median(v) == statistics.median(v)
    assert M.median([3.0, 1.0, 2.0]) == 2.0 and M.median([4.0, 1.0, 2.0, 3.0]) == 2.5


def test_speedup_by_hand():
    # test 0: medians 4 / 2 = 2; test 1: medians 3 / 6 = 0.5 -> mean 1.25
    ref = [[5.0, 4.0, 1.0], [3.0, 3.0]]
    gen = [[2.0, 9.0, 1.0], [4.0, 8.0]]
    assert M.speedup(ref, gen) == 1.25
    # the order of the repetitions does not matter; halving every generated latency doubles the speedup
    assert M.speedup([r[::-1] for r in ref], gen) == 1.25
    assert M.speedup(ref, [[x / 2 for x in g] for g in gen]) == 2.5
    assert math.isnan(M.speedup([], []))


def test_accuracies_and_verdicts_by_hand():
    call, execution = M.accuracies([1, 1, 0, 1], [1, 0, 0, 1])
    assert call == 0.75 and execution == 2 / 3
    call, execution = M.accuracies([0, 0], [0, 0])
    assert call == 0.0 and math.isnan(execution)
    rec = np.zeros((3, 2), dtype=[("pass", "<i4")])
    rec["pass"] = [[1, 1], [1, 0], [1, 1]]
    assert M.verdicts(rec).tolist() == [True, False]
    assert M.verdicts(np.zeros((0, 2), dtype=[("pass", "<i4")])).tolist() == [True, True]   # no unit test: nothing fails
