"""Exact products of FP64 data in big-integer arithmetic, and the error measures (oracle; test infrastructure).

The paper measures accuracy against a GEMM computed with 128-bit MPFR arithmetic rounded to FP64
(Section 5.3).  MPFR is not available here, and a correctly rounded reference is weaker than an
exact one anyway: every finite double is an integer times a power of two, so an inner product of
doubles is an exact rational number that Python integers hold without any rounding.

  E_AB(i,j) = |C_hat - C*| / (|A| |B|)_ij     componentwise error in the usual backward-stable-GEMM form
  E_C(i,j)  = |C_hat - C*| / |C*_ij|          relative error of the entry itself (what the paper plots for
                                              its positive inputs, where both measures coincide)
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import Iterable, List, Sequence, Tuple

import numpy as np


def int_exp(x: float) -> Tuple[int, int]:
    """x = mant * 2^exp exactly, mant a Python int (|mant| < 2^53)."""
    m, e = math.frexp(float(x))
    return int(m * (1 << 53)), e - 53


def vec_int_exp(v: np.ndarray):
    m, e = np.frexp(np.asarray(v, dtype=np.float64))
    mant = (m * float(1 << 53)).astype(np.int64)          # exact: m has at most 53 significant bits
    return [int(t) for t in mant], [int(t) - 53 for t in e]


def exact_dot(x: np.ndarray, y: np.ndarray, absolute: bool = False) -> Fraction:
    """Exact sum_k x_k y_k (or sum |x_k||y_k|) as a Fraction."""
    mx, ex = vec_int_exp(x)
    my, ey = vec_int_exp(y)
    if not mx:
        return Fraction(0)
    emin = min(a + b for a, b in zip(ex, ey))
    total = 0
    for a, b, ea, eb in zip(mx, my, ex, ey):
        pr = a * b
        if absolute and pr < 0:
            pr = -pr
        total += pr << (ea + eb - emin)
    return Fraction(total) * (Fraction(2) ** emin)


def exact_matmul(A: np.ndarray, B: np.ndarray) -> List[List[Fraction]]:
    """Exact A @ B for tiny matrices."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    return [[exact_dot(A[i, :], B[:, j]) for j in range(B.shape[1])] for i in range(A.shape[0])]


def round_fraction_to_double(fr: Fraction) -> float:
    """Nearest double, ties to even (Python's int/int true division is correctly rounded)."""
    return fr.numerator / fr.denominator


def sampled_errors(A: np.ndarray, B: np.ndarray, entries: Sequence[Tuple[int, int]], c_hat: Sequence[float]):
    """For sampled output entries (i, j) with computed values c_hat: (max E_AB, max E_C, per-entry lists)."""
    e_ab, e_c = [], []
    for (i, j), ch in zip(entries, c_hat):
        exact = exact_dot(A[i, :], B[:, j])
        scale = exact_dot(A[i, :], B[:, j], absolute=True)
        err = abs(Fraction(float(ch)) - exact)
        e_ab.append(float(err / scale) if scale != 0 else (0.0 if err == 0 else math.inf))
        e_c.append(float(err / abs(exact)) if exact != 0 else (0.0 if err == 0 else math.inf))
    return (max(e_ab) if e_ab else 0.0), (max(e_c) if e_c else 0.0), e_ab, e_c


def _veltkamp_split(v: np.ndarray):
    """v = hi + lo exactly, both with at most 26 significant bits (Veltkamp's splitting with the constant 2^27 + 1;
    numpy never fuses the multiply and the subtractions)."""
    v = np.asarray(v, dtype=np.float64)
    c = v * 134217729.0
    hi = c - (c - v)
    return hi, v - hi


def dot_residuals(x: np.ndarray, y: np.ndarray, c_hat: float):
    """(c_hat - x.y, x.y), each the EXACT value rounded once to FP64, for FP64 vectors far from overflow/underflow.

    Every product x_k y_k is the sum of four products of 26-bit halves, each exact in FP64; math.fsum adds any list of
    doubles without rounding error and rounds the final sum once.  Thousands of entries per second, where the
    big-integer route of `exact_dot` manages a few hundred; pinned against it by the tests."""
    xh, xl = _veltkamp_split(x)
    yh, yl = _veltkamp_split(y)
    parts = np.concatenate([xh * yh, xh * yl, xl * yh, xl * yl])
    if not np.all(np.isfinite(parts)):
        raise OverflowError("dot_residuals: operands too close to the overflow threshold")
    lst = parts.tolist()
    dot = math.fsum(lst)
    lst.append(-float(c_hat))
    return -math.fsum(lst), dot


def sampled_errors_fast(A: np.ndarray, B: np.ndarray, entries: Sequence[Tuple[int, int]], c_hat: Sequence[float]):
    """Like `sampled_errors`, with the residuals from `dot_residuals` (exact, rounded once) and the scale
    (|A||B|)_ij from an ordinary FP64 dot product of the absolute values (relative error ~1e-13, irrelevant for a
    ratio).  For thousands of entries at the benchmark's inner dimensions."""
    e_ab, e_c = [], []
    for (i, j), ch in zip(entries, c_hat):
        x, y = A[i, :], B[:, j]
        err, dot = dot_residuals(x, y, ch)
        err = abs(err)
        scale = float(np.abs(x) @ np.abs(y))
        e_ab.append(err / scale if scale != 0 else (0.0 if err == 0 else math.inf))
        e_c.append(err / abs(dot) if dot != 0 else (0.0 if err == 0 else math.inf))
    return (max(e_ab) if e_ab else 0.0), (max(e_c) if e_c else 0.0), e_ab, e_c


def ulp_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Number of FP64 values between a and b (0 = same bits up to the sign of zero), elementwise."""
    def key(v):
        u = np.ascontiguousarray(v, dtype=np.float64).view(np.int64)
        return np.where(u < 0, np.int64(-(2 ** 63)) - u, u)      # monotone map of the doubles onto the integers
    return np.abs(key(a).astype(object) - key(b).astype(object))


def sample_entries(m: int, n: int, count: int, seed: int = 1234) -> List[Tuple[int, int]]:
    rng = np.random.default_rng(seed)
    return [(int(i), int(j)) for i, j in zip(rng.integers(0, m, count), rng.integers(0, n, count))]
