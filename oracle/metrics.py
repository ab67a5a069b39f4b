"""Plain statements of the evaluation metrics that consume the check's verdicts.  TEST INFRASTRUCTURE ONLY.

GEAK section "Evaluation Metrics" (call accuracy, execution accuracy, speedup) and section 4.2
(parallel scaling: accuracy is estimated with pass@k).  The paper gives the speedup in words and no
formula for pass@k; the readings:

  M1  a kernel is correct iff it satisfies ALL unit tests (section 3.3): the verdict of candidate k
      is the AND of the pass flags of its (segment, candidate) records.
  M2  call accuracy = kernels that compile and run / all kernels;
      execution accuracy = kernels that satisfy all unit tests / kernels that compile (NaN if none does).
  M3  speedup of a correct kernel = mean over unit tests of
      median(reference latencies of the test) / median(generated latencies of the test);
      the median of an even number of values is the mean of the two middle ones; the mean over the
      tests is accumulated in test order, in binary64.
  M4  pass@k from n samples of which c are correct = 1 - C(n - c, k) / C(n, k), the probability that a
      uniformly drawn k-subset of the samples holds a correct one (the usual unbiased estimator); k <= n.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np


def verdicts(records: np.ndarray) -> np.ndarray:
    """M1: records of shape (segments, candidates) with a 'pass' field -> bool array (candidates,)."""
    out = np.ones(records.shape[1], dtype=bool)
    for s in range(records.shape[0]):
        for k in range(records.shape[1]):
            if int(records[s, k]["pass"]) == 0:
                out[k] = False
    return out


def accuracies(compiled, correct):
    """M2: two sequences of booleans of equal length -> (call accuracy, execution accuracy)."""
    compiled = [bool(x) for x in compiled]
    correct = [bool(x) for x in correct]
    n = len(compiled)
    n_compiled = sum(compiled)
    n_correct = sum(1 for a, b in zip(compiled, correct) if a and b)
    call = n_compiled / n if n else float("nan")
    execution = n_correct / n_compiled if n_compiled else float("nan")
    return call, execution


def median(values) -> float:
    v = sorted(float(x) for x in values)
    n = len(v)
    if n == 0:
        return float("nan")
    if n % 2:
        return v[n // 2]
    return 0.5 * (v[n // 2 - 1] + v[n // 2])


def speedup(ref_latencies, gen_latencies) -> float:
    """M3: two sequences (one entry per unit test) of sequences of repeated latencies."""
    if len(ref_latencies) != len(gen_latencies) or not len(ref_latencies):
        return float("nan")
    total = 0.0
    for r, g in zip(ref_latencies, gen_latencies):
        total = total + median(r) / median(g)
    return total / len(ref_latencies)


def pass_at_k(n: int, c: int, k: int) -> Fraction:
    """M4, exactly."""
    if not (0 <= c <= n and 1 <= k <= n):
        raise ValueError("need 0 <= c <= n and 1 <= k <= n")
    return 1 - Fraction(math.comb(n - c, k), math.comb(n, k))
