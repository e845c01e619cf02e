"""Seeded synthetic input generators shared by the tests, the benchmark and the oracle checks.

This module holds no arithmetic of the Ozaki scheme: it only draws matrices.

The recipe is the phi-parametrised test matrix used in the Ozaki-scheme literature,
    a = (u - 0.5) * exp(phi * z),   u ~ U(0,1),  z ~ N(0,1),
which gives zero-mean entries whose magnitudes are log-normally spread; a larger phi
widens the exponent range inside every row/column and therefore raises the number of
slices the scheme needs.  The paper's own evaluation (Section 5.1) uses U(1,10) instead;
`uniform_1_10` provides that recipe for the Table 2 style experiments.
"""
from __future__ import annotations

import numpy as np


def phi_matrix(rows: int, cols: int, phi: float, rng: np.random.Generator) -> np.ndarray:
    """rows x cols float64 matrix (C order) with entries (u-0.5)*exp(phi*z)."""
    u = rng.random((rows, cols))
    z = rng.standard_normal((rows, cols))
    z *= phi
    np.exp(z, out=z)
    u -= 0.5
    u *= z
    return u


def phi_pair(m: int, n: int, k: int, phi: float, seed: int = 0):
    """A (m x k) and B (k x n) drawn in that order from numpy.random.default_rng(seed)."""
    rng = np.random.default_rng(seed)
    A = phi_matrix(m, k, phi, rng)
    B = phi_matrix(k, n, phi, rng)
    return A, B


def uniform_1_10(rows: int, cols: int, rng: np.random.Generator) -> np.ndarray:
    """Entries uniform in (1, 10): the input of the paper's Section 5.1."""
    return 1.0 + 9.0 * rng.random((rows, cols))


def full_mantissa_one_binade(rows: int, cols: int, rng: np.random.Generator) -> np.ndarray:
    """Entries in [1, 2) whose 52 fraction bits are random with the last bit forced to 1:
    every one of the 53 significand bits carries information (the premise of Table 2)."""
    frac = rng.integers(0, 1 << 52, size=(rows, cols), dtype=np.uint64) | np.uint64(1)
    bits = frac | np.uint64(0x3FF0000000000000)
    return bits.view(np.float64)


def nasty_rows(rng: np.random.Generator, rows: int, k: int) -> np.ndarray:
    """rows x k matrix (rows >= 9) whose first nine rows are the corner cases of the slicing step: a zero vector, a
    maximum that is a power of two, one just above a power of two, a row that needs a single slice, a half-empty row, a
    row with one entry 2^300 times the rest, a full-significand one-binade row with random signs, a row scaled down by
    2^-400, and a row of exact ties of the first slice's rounding; the other rows are phi = 3 entries."""
    X = phi_matrix(rows, k, 3.0, rng)
    X[0, :] = 0.0                                     # zero vector: c := 0
    X[1, :] = 1.0                                     # max is a power of two
    X[2, :] = np.nextafter(1.0, 2.0)                  # just above a power of two
    X[3, :] = np.ldexp(rng.integers(-16, 17, k).astype(np.float64), -3)   # one-slice row
    X[4, : k // 2] = 0.0
    X[5, 0] = 2.0 ** 300
    X[6, :] = full_mantissa_one_binade(1, k, rng)[0] * np.where(rng.random(k) < 0.5, -1, 1)
    X[7, :] *= 2.0 ** -400
    # ties: entries exactly half way between two slice values of the first slice
    X[8, :] = 0.0
    X[8, 0] = 1.0
    X[8, 1:9] = (2 * np.arange(8) + 1) / 32.0         # odd multiples of 2^-5 when the first ulp is 2^-4
    return X


#: The benchmark configurations: name -> shape, phi, slice format, k_block (0 = no blocking), accumulation mode.
CONFIGS = {
    "c1_256_fp8_hw":        dict(m=256,   n=256,   k=256,   phi=0.5, fmt="fp8",  k_block=0,    accum="hw"),
    "c2_4096_fp8_hw":       dict(m=4096,  n=4096,  k=4096,  phi=1.0, fmt="fp8",  k_block=0,    accum="hw"),
    "c3_8192_fp8_emu":      dict(m=8192,  n=8192,  k=8192,  phi=4.0, fmt="fp8",  k_block=0,    accum="emu"),
    "c4_16384_fp16_kb1024": dict(m=16384, n=16384, k=16384, phi=1.0, fmt="fp16", k_block=1024, accum="hw"),
    "c4_16384_fp16_kb4096": dict(m=16384, n=16384, k=16384, phi=1.0, fmt="fp16", k_block=4096, accum="hw"),
    "c4_16384_fp8":         dict(m=16384, n=16384, k=16384, phi=1.0, fmt="fp8",  k_block=0,    accum="hw"),
    "c5a_16384x1024_fp8":   dict(m=16384, n=16384, k=1024,  phi=2.0, fmt="fp8",  k_block=1024, accum="emu"),
    "c5b_1024x65536_fp8":   dict(m=1024,  n=1024,  k=65536, phi=2.0, fmt="fp8",  k_block=8192, accum="emu"),
}

#: The paper's own workload (Section 5.1): square matrices with entries uniform in (1, 10), every one of the s^2 slice
#: pairs multiplied, s = the slice count behind Table 2 for the block length (11 for FP8; 7 for FP16 with 1024-element
#: blocks), which brings the result to the correctly rounded product on the calibration sample.
PAPER_CONFIGS = {}
PAPER_NUM_SLICES = {}
for _n in (1024, 2048, 4096, 8192, 16384):
    PAPER_CONFIGS[f"paper_u110_n{_n}_fp8"] = dict(m=_n, n=_n, k=_n, dist="u110", fmt="fp8", k_block=0, accum="hw", pairs="all")
    PAPER_NUM_SLICES[f"paper_u110_n{_n}_fp8"] = 11
    PAPER_CONFIGS[f"paper_u110_n{_n}_fp16_kb1024"] = dict(m=_n, n=_n, k=_n, dist="u110", fmt="fp16", k_block=1024, accum="hw",
                                                          pairs="all")
    PAPER_NUM_SLICES[f"paper_u110_n{_n}_fp16_kb1024"] = 7


def config_pair(cfg: dict, seed: int = 0):
    """A (m x k) and B (k x n) of a configuration: the phi recipe, or uniform (1, 10) where it says dist="u110"."""
    if cfg.get("dist", "phi") == "u110":
        rng = np.random.default_rng(seed)
        return uniform_1_10(cfg["m"], cfg["k"], rng), uniform_1_10(cfg["k"], cfg["n"], rng)
    return phi_pair(cfg["m"], cfg["n"], cfg["k"], cfg["phi"], seed=seed)


#: Slices per configuration for full FP64 accuracy (error no larger than a plain FP64 GEMM on the same
#: entries): the s_native column of tests/golden/slices_per_config.txt.  S_BOUND is the smallest count
#: that meets the componentwise bound 4 k 2^-53.
NUM_SLICES = {
    "c1_256_fp8_hw": 12, "c2_4096_fp8_hw": 13, "c3_8192_fp8_emu": 16,
    "c4_16384_fp16_kb1024": 8, "c4_16384_fp16_kb4096": 9, "c4_16384_fp8": 13,
    "c5a_16384x1024_fp8": 13, "c5b_1024x65536_fp8": 13,
}
#: the same for INT8 slices (b = 6: seven bits of progress per slice instead of five), lines "<config>@int8" of the fixture
NUM_SLICES_INT8 = {
    "c1_256_fp8_hw": 9, "c2_4096_fp8_hw": 9, "c3_8192_fp8_emu": 11, "c4_16384_fp8": 9,
    "c5a_16384x1024_fp8": 9, "c5b_1024x65536_fp8": 10,
}
S_BOUND = {
    "c1_256_fp8_hw": 10, "c2_4096_fp8_hw": 10, "c3_8192_fp8_emu": 13,
    "c4_16384_fp16_kb1024": 6, "c4_16384_fp16_kb4096": 7, "c4_16384_fp8": 9,
    "c5a_16384x1024_fp8": 11, "c5b_1024x65536_fp8": 10,
}
