"""The library's host-side evaluation metrics against the oracle's (no GPU needed): speedup and
accuracies bit for bit (same operations in the same order), pass@k within the rounding of its
product form."""
import math

import numpy as np
import pytest

from oracle import metrics as M
from paper_2507_23194_amd import binding as B


@pytest.fixture(scope="module")
def lib():
    return B.library()


def test_speedup_matches_oracle_bit_for_bit(lib):
    rng = np.random.default_rng(0)
    for tests, r_ref, r_gen in [(1, 1, 1), (3, 5, 7), (17, 10, 10), (40, 4, 9), (5, 2, 2)]:
        ref = rng.lognormal(size=(tests, r_ref))
        gen = rng.lognormal(size=(tests, r_gen))
        gen[0, :] = gen[0, 0]                                 # ties
        st, got = B.geak_metrics_speedup(ref, gen)
        assert st == B.GEAK_OK and got == M.speedup(ref.tolist(), gen.tolist())
    st, got = B.geak_metrics_speedup(np.zeros((0, 3)), np.zeros((0, 3)))
    assert st == B.GEAK_OK and math.isnan(got)


def test_accuracy_matches_oracle(lib):
    rng = np.random.default_rng(1)
    for n in (1, 2, 9, 1000):
        compiled = rng.random(n) < 0.7
        correct = rng.random(n) < 0.5
        st, call, execution = B.geak_metrics_accuracy(compiled, correct)
        want = M.accuracies(compiled, correct)
        assert st == B.GEAK_OK and call == want[0]
        assert execution == want[1] or (math.isnan(execution) and math.isnan(want[1]))
    st, call, execution = B.geak_metrics_accuracy([0, 0, 0], [1, 1, 1])
    assert call == 0.0 and math.isnan(execution)


def test_pass_at_k_within_rounding_of_the_exact_value(lib):
    for n, c, k in [(1, 0, 1), (1, 1, 1), (10, 3, 1), (10, 3, 5), (10, 8, 3), (100, 1, 100), (200, 17, 10),
                    (1000, 3, 50), (100000, 12345, 7), (64, 64, 64), (64, 0, 64)]:
        st, got = B.geak_metrics_pass_at_k(n, c, k)
        exact = M.pass_at_k(n, c, k)
        assert st == B.GEAK_OK
        # c factors, each rounded twice, then one subtraction: the miss probability carries a relative error
        # of at most about 3c units in the last place
        assert abs(got - float(exact)) <= (3 * c + 2) * 2.0 ** -53, (n, c, k, got, float(exact))
    for bad in [(3, 4, 1), (3, 1, 0), (3, 1, 4)]:
        assert B.geak_metrics_pass_at_k(*bad)[0] == B.GEAK_EINVAL
