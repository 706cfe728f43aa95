"""TEST INFRASTRUCTURE -- plain CPU oracle for the per-cycle aggregation of the gradient
statistics (paper: System Architecture, temporal aggregation of metrics over k consecutive
iterations; Problem Formulation, "State representation": sigma_norm and sigma_norm^2 enter the
state; "Reward function design": penalty -eta (sigma_norm^2 + sigma_norm) for adaptive optimizers
and batch size regulariser -delta (log2 BatchSize - 5)).

The paper does not say how the k iterations are combined; the reading taken is the arithmetic
mean of every entry of the statistics record over the cycle, plus "pooled" ratios formed from the
mean sums (mean T over mean A), which is how the noise-scale literature averages before dividing.  The reading itself has nothing
in the paper to be checked against (parity against the paper: unpinned); its arithmetic is pinned
against numpy.mean, single-iteration and identical-iteration cases and closed forms.
Plain float64 numpy, one iteration after the other in call order.  Shares nothing with the HIP
path.
"""
import math

import numpy as np

HEAD = 8
EXTRA = 4


def summary_count(K, S):
    return (1 + S) * (HEAD + 2 * K + EXTRA) + K


def cycle_summary(stats_list, K, S, batch_sizes, eta, delta):
    """stats_list: the k statistics arrays of one cycle, each float64[1+S, 8+2K], in call order.
    Returns float64[summary_count(K, S)]."""
    R = HEAD + 2 * K
    k_iters = len(stats_list)
    assert k_iters >= 1
    total = np.zeros((1 + S, R), dtype=np.float64)
    for st in stats_list:                       # running sum in call order
        total = total + np.asarray(st, dtype=np.float64).reshape(1 + S, R)
    mean = total / float(k_iters)
    B = float(sum(int(x) for x in batch_sizes))
    out = np.zeros(summary_count(K, S), dtype=np.float64)
    for r in range(1 + S):
        base = r * (R + EXTRA)
        out[base:base + R] = mean[r]
        A, T = mean[r, 0], mean[r, 1]
        with np.errstate(all="ignore"):
            out[base + R + 0] = np.float64(T) / (np.float64(A) - np.float64(T) / B)
            s2 = np.float64(T) / (B * np.float64(A))
        out[base + R + 1] = s2
        out[base + R + 2] = math.sqrt(s2) if s2 > 0 else 0.0
        out[base + R + 3] = -eta * (mean[r, 5] + mean[r, 6])
    tail = (1 + S) * (R + EXTRA)
    for k in range(K):
        out[tail + k] = -delta * (math.log2(float(batch_sizes[k])) - 5.0)
    return out
