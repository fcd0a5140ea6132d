"""Oracle (test infrastructure): per-head kept rank from the singular-value removal rate.

Section 5.2, Eq. (1): with singular values theta_0 >= theta_1 >= ... of a head
and a removal rate r shared by all heads, the last kept dimension j satisfies

    sum_{i > j} theta_i / sum_i theta_i  <=  r  <  sum_{i >= j} theta_i / sum_i theta_i

i.e. the removed dimensions j+1 .. d_h-1 carry at most a fraction r of the
total singular-value mass and removing dimension j as well would exceed it.
The compression rate p is tied to j by j = floor((1 - p)(d_h - 1)). The
superscript on theta is an index, not a power.

Readings: the kept rank is j + 1; r >= 1 keeps one dimension (j = 0); the rank
handed to the kernels is rounded up to a multiple of 16 (implementation
paragraph of Section 6.1).
"""
from __future__ import annotations

import numpy as np


def last_kept_index(theta, r: float) -> int:
    """j of Eq. (1): the largest j whose tail sum_{i >= j} theta_i / total exceeds r.

    The tails are accumulated in float64 from the last dimension backwards,
    tail_j = tail_{j+1} + theta_j, total = tail_0, and the test is written without the division,
    tail_j > r * total, so that the decision is reproducible operation by operation.
    """
    theta = [float(t) for t in np.asarray(theta, dtype=np.float64)]
    n = len(theta)
    tails = [0.0] * (n + 1)
    for j in range(n - 1, -1, -1):
        tails[j] = tails[j + 1] + theta[j]
    total = tails[0]
    j_found = 0
    for j in range(n):
        if tails[j] > float(r) * total:
            j_found = j
    return j_found


def kept_rank(theta, r: float, multiple: int = 16) -> int:
    k = last_kept_index(theta, r) + 1
    return -(-k // multiple) * multiple


def compression_rate_interval(j: int, d_h: int):
    """All p with j = floor((1 - p)(d_h - 1)): p in (1 - (j+1)/(d_h-1), 1 - j/(d_h-1)]."""
    return 1.0 - (j + 1) / (d_h - 1), 1.0 - j / (d_h - 1)
