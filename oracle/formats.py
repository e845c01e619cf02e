"""Type2 storage formats of the slices (oracle side; test infrastructure).

The paper stores each slice in the input format of the matrix unit ("Type2", Section 3):
FP8 E4M3 or FP16 (Section 4.1).  The conversion cvt_Type2 of Eq. 8 is exact by
construction of the slices, so "encoding" here means: find the code whose value IS the
given number, and fail loudly if there is none.

FP8 E4M3 follows the OCP 8-bit floating point definition (1 sign, 4 exponent bits with
bias 7, 3 fraction bits, no infinities, S.1111.111 is NaN, largest finite value 448),
which is the flavour the gfx950 matrix unit consumes.

FP6 E2M3 (Section 4.1 names FP6 as the format to try where it is twice as fast as FP8) is the
OCP microscaling element format: 1 sign, 2 exponent bits with bias 1, 3 fraction bits, no
infinities or NaNs; subnormals 0.125 .. 0.875, normals 1.0 .. 7.5.  It has the same four
significand bits as E4M3, so the slices themselves are the same numbers q * 2^-b; but its
smallest step is 1/8, so the stored code holds TWICE the value of Eq. 8 (q * 2^-(b-1), at
most 2.0) and the factor 1/4 per product is applied with the exponents.
"""
from __future__ import annotations

import numpy as np

#: significand bits including the hidden bit (the paper's m_Type2, Section 3).  "int8" is the comparison path on the
#: integer matrix unit (the variant of the scheme Section 2 cites): a two's-complement byte holds the integers
#: -128 .. 127, so the symmetric range |q| <= 2^b of Eq. 5-8 fits for b <= 6.
SIGNIFICAND_BITS = {"fp8": 4, "fp16": 11, "fp6": 4, "fp6_e3m2": 3, "int8": 6}

#: significand bits of the accumulator type (the paper's m_Type3): FP32, or INT32 for int8 slices.  An INT32 sum is
#: exact up to 2^31 - 1 in magnitude, one short of the power of two Eq. 1 is written for, hence EXACT_WINDOW.
ACCUMULATOR_BITS = {"fp8": 24, "fp16": 24, "fp6": 24, "fp6_e3m2": 24, "int8": 31}

#: largest magnitude, in units of the product of two slice units, that the matrix unit accumulates exactly
EXACT_WINDOW = {"fp8": 1 << 24, "fp16": 1 << 24, "fp6": 1 << 24, "fp6_e3m2": 1 << 24, "int8": (1 << 31) - 1}

#: the stored code holds slice * 2^CODE_SHIFT (nonzero only for FP6 E2M3, see above)
CODE_SHIFT = {"fp8": 0, "fp16": 0, "fp6": 1, "fp6_e3m2": 0, "int8": 0}


def e4m3_decode_table() -> np.ndarray:
    """Value of each of the 256 OCP E4M3 byte codes (NaN codes -> nan)."""
    vals = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        f = code & 0x7
        if e == 0xF and f == 0x7:
            vals[code] = np.nan
        elif e == 0:
            vals[code] = sign * (f / 8.0) * 2.0 ** (1 - 7)          # subnormal
        else:
            vals[code] = sign * (1.0 + f / 8.0) * 2.0 ** (e - 7)    # normal
    return vals


_E4M3_VALUES = e4m3_decode_table()


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    return _E4M3_VALUES[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode_exact(values: np.ndarray) -> np.ndarray:
    """Byte codes of `values`; every value must be exactly representable.  Zero (of either
    sign) encodes as 0x00: the scheme never distinguishes the sign of a zero slice entry."""
    values = np.asarray(values, dtype=np.float64)
    finite_codes = np.array([c for c in range(256) if not np.isnan(_E4M3_VALUES[c]) and c != 0x80], dtype=np.uint8)
    table_vals = _E4M3_VALUES[finite_codes]
    order = np.argsort(table_vals, kind="stable")
    sorted_vals = table_vals[order]
    sorted_codes = finite_codes[order]
    pos = np.searchsorted(sorted_vals, values.ravel())
    pos = np.clip(pos, 0, len(sorted_vals) - 1)
    if not np.array_equal(sorted_vals[pos], values.ravel()):
        bad = values.ravel()[sorted_vals[pos] != values.ravel()]
        raise ValueError(f"value not representable in FP8 E4M3: {bad[:4]}")
    return sorted_codes[pos].reshape(values.shape)


def fp16_encode_exact(values: np.ndarray) -> np.ndarray:
    """IEEE binary16 bit patterns (uint16) of `values`; every value must be exactly representable."""
    values = np.asarray(values, dtype=np.float64)
    h = values.astype(np.float16)
    if not np.array_equal(h.astype(np.float64), values):
        raise ValueError("value not representable in FP16")
    h = np.where(h == 0, np.float16(0.0), h)      # +0 for either zero
    return h.view(np.uint16)


def fp16_decode(codes: np.ndarray) -> np.ndarray:
    return np.asarray(codes, dtype=np.uint16).view(np.float16).astype(np.float64)


def e2m3_decode_table() -> np.ndarray:
    """Value of each of the 64 OCP E2M3 codes."""
    vals = np.empty(64, dtype=np.float64)
    for code in range(64):
        sign = -1.0 if code & 0x20 else 1.0
        e = (code >> 3) & 0x3
        f = code & 0x7
        if e == 0:
            vals[code] = sign * (f / 8.0) * 2.0 ** (1 - 1)          # subnormal
        else:
            vals[code] = sign * (1.0 + f / 8.0) * 2.0 ** (e - 1)    # normal
    return vals


_E2M3_VALUES = e2m3_decode_table()


def e2m3_decode(codes: np.ndarray) -> np.ndarray:
    return _E2M3_VALUES[np.asarray(codes, dtype=np.uint8)]


def e2m3_encode_exact(values: np.ndarray) -> np.ndarray:
    """6-bit codes (one per uint8) of `values`; every value must be exactly representable; zero -> 0."""
    values = np.asarray(values, dtype=np.float64)
    out = np.zeros(values.shape, dtype=np.uint8)
    found = values == 0
    for code in range(64):
        if code in (0x00, 0x20):
            continue
        hit = values == _E2M3_VALUES[code]
        out[hit] = code
        found |= hit
    if not found.all():
        raise ValueError(f"value not representable in FP6 E2M3: {values[~found].ravel()[:4]}")
    return out


def e3m2_decode_table() -> np.ndarray:
    """Value of each of the 64 OCP E3M2 codes (1 sign, 3 exponent bits with bias 3, 2 fraction bits, no Inf/NaN):
    the FP6 flavour of the paper's Table 2."""
    vals = np.empty(64, dtype=np.float64)
    for code in range(64):
        sign = -1.0 if code & 0x20 else 1.0
        e = (code >> 2) & 0x7
        f = code & 0x3
        if e == 0:
            vals[code] = sign * (f / 4.0) * 2.0 ** (1 - 3)          # subnormal
        else:
            vals[code] = sign * (1.0 + f / 4.0) * 2.0 ** (e - 3)    # normal
    return vals


_E3M2_VALUES = e3m2_decode_table()


def e3m2_decode(codes: np.ndarray) -> np.ndarray:
    return _E3M2_VALUES[np.asarray(codes, dtype=np.uint8)]


def e3m2_encode_exact(values: np.ndarray) -> np.ndarray:
    values = np.asarray(values, dtype=np.float64)
    out = np.zeros(values.shape, dtype=np.uint8)
    found = values == 0
    for code in range(64):
        if code in (0x00, 0x20):
            continue
        hit = values == _E3M2_VALUES[code]
        out[hit] = code
        found |= hit
    if not found.all():
        raise ValueError(f"value not representable in FP6 E3M2: {values[~found].ravel()[:4]}")
    return out


def int8_encode_exact(values: np.ndarray, b: int) -> np.ndarray:
    """Two's-complement bytes of the integers q = values * 2^b; every q must be an integer in [-128, 127]."""
    q = np.ldexp(np.asarray(values, dtype=np.float64), b)
    if not np.array_equal(q, np.rint(q)) or (q.size and (q.min() < -128 or q.max() > 127)):
        raise ValueError("slice entry is not an INT8 integer")
    return q.astype(np.int8).view(np.uint8)


def int8_decode(codes: np.ndarray, b: int) -> np.ndarray:
    return np.ldexp(np.asarray(codes, dtype=np.uint8).view(np.int8).astype(np.float64), -b)


def encode_exact(fmt: str, values: np.ndarray, b: int = None) -> np.ndarray:
    """Codes of the slice values `values` (= q * 2^-b, Eq. 8) in format `fmt` (b is needed for "int8" only)."""
    if fmt == "int8":
        return int8_encode_exact(values, b)
    if fmt == "fp6":
        return e2m3_encode_exact(np.asarray(values, dtype=np.float64) * 2.0 ** CODE_SHIFT["fp6"])
    if fmt == "fp6_e3m2":
        return e3m2_encode_exact(values)
    if fmt == "fp8":
        return e4m3_encode_exact(values)
    if fmt == "fp16":
        return fp16_encode_exact(values)
    raise ValueError(fmt)


def decode(fmt: str, codes: np.ndarray, b: int = None) -> np.ndarray:
    """Slice values (= q * 2^-b) of the codes."""
    if fmt == "int8":
        return int8_decode(codes, b)
    if fmt == "fp6":
        return e2m3_decode(codes) * 2.0 ** -CODE_SHIFT["fp6"]
    if fmt == "fp6_e3m2":
        return e3m2_decode(codes)
    if fmt == "fp8":
        return e4m3_decode(codes)
    if fmt == "fp16":
        return fp16_decode(codes)
    raise ValueError(fmt)
