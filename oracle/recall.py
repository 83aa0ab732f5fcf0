"""Expected recall of bucketed approximate top-k (Appendix C, "Recall model").

TEST INFRASTRUCTURE ONLY (see the package docstring).

Recall R(k, b, k_b) = Z / k, where Z counts how many of the true top-k elements the
bucketed method returns.
"""
from __future__ import annotations

import math

from scipy import stats


def expected_recall_eq1(k: int, b: int, k_b: int) -> float:
    """Appendix C, Eq. 1:  E[R] = (k_b + sum_{i=k_b}^{k-1} F(k_b - 1; i, 1/b)) / k.

    F(x; i, p) is the Binomial(i, p) CDF.  Derived for inputs whose top-k positions
    fall into buckets uniformly and independently, with k_b much smaller than n/b.
    """
    total = float(k_b)
    for i in range(k_b, k):
        total += stats.binom.cdf(k_b - 1, i, 1.0 / b)
    return total / k


def expected_recall_kb1(k: int, b: int) -> float:
    """Appendix C, the k_b = 1 special case printed below Eq. 1:  (b/k)(1 - ((b-1)/b)^k)."""
    return (b / k) * (1.0 - ((b - 1.0) / b) ** k)


def expected_recall_iid_exact(n: int, k: int, b: int, k_b: int) -> float:
    """Exact expectation for i.i.d. continuous inputs, without the k_b << n/b assumption.

    Not printed in the paper; it is the remark after Eq. 1 (dropping k_b << n/b makes
    Eq. 1 a bound) made precise.  The positions of the true top-k form a uniform random
    k-subset of the n positions, bucket j holds len_j of them, so the number of true
    top-k elements in bucket j is Hypergeometric(n, len_j, k), of which min(., k_b) are
    returned.  Linearity of expectation gives  E[Z] = sum_j E[min(H_j, k_b)].
    """
    total = 0.0
    by_len = {}
    for j in range(b):
        length = (n - j + b - 1) // b
        by_len[length] = by_len.get(length, 0) + 1
    for length, count in by_len.items():
        h = stats.hypergeom(n, length, k)
        e = 0.0
        for z in range(0, min(length, k) + 1):
            e += min(z, k_b) * h.pmf(z)
        total += count * e
    return total / k


def worst_case_recall(n: int, k: int, b: int, k_b: int) -> float:
    """Appendix C, Eq. 2: all true top-k elements packed into as few buckets as possible.

    R_wc = (floor(b k / n) k_b + min(k_b, k mod (n/b))) / k, for b dividing n.
    """
    if n % b:
        raise ValueError("Eq. 2 is stated for b dividing n")
    length = n // b
    return (math.floor(b * k / n) * k_b + min(k_b, k % length)) / k
