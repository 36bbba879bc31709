"""TEST INFRASTRUCTURE - the Unified Metric of Section 4.5 (Eq. 16-20) in plain numpy float64.

For one activation layer and one candidate approximation function:
    Q = quantization sensitivity, the SQNR in dB between the layer's real-valued output X and
        the candidate's dequantized output X^                                    (Eq. 18)
    P = quantization perturbation ||X - X^||_2^2                                  (Eq. 19)
    C = integer operation count of the layer                                      (Eq. 20)
    N(x) = log(1 + exp(x))  (Softplus)                                            (Eq. 17)
    score = 3 / (1 / N(Q) + N(P) + N(C)); the candidate with the highest score is assigned to
    the layer, and Omega is the sum of the assigned scores over the layers       (Eq. 16)

Readings (the paper is at odds with itself or silent; each is declared):
  * Eq. 18 prints "20 log" of the POWER ratio, but the worked example of the same section
    (signal power 10^4; error powers 100 and 60 -> 20 dB and 22.21 dB) is 10 log10 of the power
    ratio (= 20 log10 of the amplitude ratio).  The example decides: Q = 10 log10(E[X^2] / E[(X - X^)^2]).
  * "log" of Eq. 17 is the natural logarithm (Softplus).
  * The operation counts are this build's count of the arithmetic and bit operations of each
    step of Section 4.3 / 4.4 per element (table below); the paper prints none.
  * mode "per_element": P and C divided by the element count.  Literally (mode "literal"),
    P and C of a whole layer are 10^3 .. 10^9, N(P) + N(C) = P + C swamps 1 / N(Q) and the
    cheapest candidate always wins; the normalisation the paper uses is not printed.

Only tests may import this module; it shares nothing with the HIP library's host code.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Sequence

import numpy as np

# integer operations per element, counted from the steps of the method (reductions once per
# element; the one division per row of Eq. 15 is added per row)
SOFTMAX_OPS_COMMON = (2      # Eq. 6: compare for the row maximum, subtract it
                      + 4    # Eq. 7: two shifts, one add, one subtract
                      + 4    # Eq. 8: negate, divide by i0, multiply and subtract for the remainder
                      + 2    # Eq. 9: shift left by N, shift right by q
                      + 1    # row sum
                      + 2)   # Eq. 15: multiply by the row factor, shift
SOFTMAX_OPS_FRACTION = {0: 3,    # Eq. 10: negate, shift, add 1/S
                        1: 7,    # Eq. 13-14: negate, three shifts, two adds, add 1/S
                        2: 10}   # second-degree term on top: square, divide, add
SOFTMAX_OPS_PER_ROW = 1          # floor(2^M / sum)
GELU_OPS = {0: 17,   # centre, sign, abs, min, add b, square, add 1, times sign, add 1, shift, times x,
                     # requantization (multiply, add, shift, add zero-point, two clamps)
            1: 18}   # the quartic reuses the square: one more multiply


def softmax_op_count(variant: int, rows: int, cols: int) -> int:
    return rows * cols * (SOFTMAX_OPS_COMMON + SOFTMAX_OPS_FRACTION[variant]) + rows * SOFTMAX_OPS_PER_ROW


def gelu_op_count(variant: int, n: int) -> int:
    return n * GELU_OPS[variant]


def softplus(x: float) -> float:
    """log(1 + exp(x)) (Eq. 17), written so that exp never overflows: the two branches are the
    same function."""
    if x == math.inf:
        return math.inf
    return x + math.log1p(math.exp(-x)) if x > 0 else math.log1p(math.exp(x))


def sqnr_db(x: np.ndarray, x_hat: np.ndarray) -> float:
    """Eq. 18 under the reading above; +inf when the two agree exactly."""
    x = np.asarray(x, np.float64).ravel()
    e = x - np.asarray(x_hat, np.float64).ravel()
    signal, noise = float(np.mean(x * x)), float(np.mean(e * e))
    if noise == 0.0:
        return math.inf
    if signal == 0.0:
        return -math.inf
    return 10.0 * math.log10(signal / noise)


def perturbation(x: np.ndarray, x_hat: np.ndarray) -> float:
    e = np.asarray(x, np.float64).ravel() - np.asarray(x_hat, np.float64).ravel()
    return float(np.sum(e * e))                                        # Eq. 19


@dataclass
class Terms:
    q_db: float
    p: float
    c: float
    score: float


def unified_metric(x, x_hat, op_count: float, mode: str = "literal") -> Terms:
    n = int(np.asarray(x).size)
    q = sqnr_db(x, x_hat)
    p = perturbation(x, x_hat)
    c = float(op_count)
    if mode == "per_element":
        p, c = p / n, c / n
    elif mode != "literal":
        raise ValueError(mode)
    nq = softplus(q)
    inv_nq = 0.0 if nq == math.inf else (math.inf if nq == 0.0 else 1.0 / nq)
    score = 3.0 / (inv_nq + softplus(p) + softplus(c))                 # Eq. 16, one layer
    return Terms(q, p, c, score)


def select(candidates: Sequence[Terms]) -> int:
    """Index of the candidate with the highest score (the first one among equals)."""
    best = 0
    for i, t in enumerate(candidates):
        if t.score > candidates[best].score:
            best = i
    return best


def omega(assigned_scores: Sequence[float]) -> float:
    return float(sum(assigned_scores))                                 # Eq. 16
