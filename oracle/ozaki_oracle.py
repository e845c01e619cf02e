"""Ozaki-scheme DGEMM, step by step, in plain numpy FP64 (oracle; test infrastructure).

Follows the paper's Section 3 in its order and notation:

  constants   gamma, xi, rho                      Eq. 1-3
  slicing     c, sigma, v, x^(p+1), slice         Eq. 4-8 (literal FP64 arithmetic, numpy never fuses a*b+c)
  products    slice-pair inner products           Eq. 10-11 (exact; here exact integers)
  accumulate  sum of 2^(c_x+c_y) * product        Eq. 10, in Type1 = FP64 arithmetic (Section 3, last paragraphs)
  blocking    the above per block of the inner dimension, block results summed in FP64   Section 4.3

Conventions (where the paper leaves a point open, the reading taken is stated here):
  * A is m x k, B is k x n, both given as ordinary numpy arrays (logical indexing A[i, kk], B[kk, j]).
  * Slices of A are taken per row of A, slices of B per column of B, over one k-block at a time.
  * b = 53 - rho is the number of magnitude bits of a slice entry: entry = q * 2^-b, q integer, |q| <= 2^b.
  * Eq. 4's ceil(log2(max)) is evaluated exactly: the smallest integer c with max <= 2^c; c = 0 for a zero vector.
  * With num_slices = s on both operands the pairs used are those with p + q <= s + 1 ("triangle"),
    or all s*s ("full").  Accumulation order: anti-diagonals g = p+q from the largest g (smallest
    magnitude) down to 2, p ascending inside an anti-diagonal.
  * Accumulation (the paper says only that it is done in Type1 arithmetic and that its order was tuned):
    the DEFINITION here is `accumulate="plain"`: the terms 2^(c_x+c_y) * product of Eq. 10 are added one
    by one, each addition rounded to FP64, in the order above.  Two named variants exist beside it, both
    readings of the same passage that a device may implement instead, each with the same order:
    "runs" adds consecutive terms of one anti-diagonal that share their power-of-two scale exactly before
    the one rounded addition; "exact" sums all terms of a block in a wide fixed-point integer and rounds
    once (see `block_result`).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, List, Sequence, Tuple

import numpy as np

from . import formats

M_TYPE1 = 53          # FP64 significand bits (hidden bit included)
M_FP32 = 24
M_FP16 = 11


# --------------------------------------------------------------------------------------
# Eq. 1-3
# --------------------------------------------------------------------------------------
def gamma_const(k: int, m_type3: int = M_FP32, m_type1: int = M_TYPE1) -> int:
    """Eq. 1: gamma = ceil(m1 - (m3 - log2 k)/2), evaluated without floating point:
    m1 - gamma = floor((m3 - log2 k)/2) is the largest integer t with k * 4^t <= 2^m3."""
    if k < 1:
        raise ValueError("k must be positive")
    def fits(t: int) -> bool:          # k * 4^t <= 2^m3, in integers, for t of either sign
        if t >= 0:
            return (k << (2 * t)) <= (1 << m_type3)
        return k <= (1 << (m_type3 - 2 * t))

    t = m_type3                        # generous start, walk down to the largest t that fits
    while not fits(t):
        t -= 1
    return m_type1 - t


def xi_const(m_type2: int, m_type1: int = M_TYPE1) -> int:
    """Eq. 2."""
    return m_type1 - m_type2


def rho_const(k: int, m_type2: int, m_type3: int = M_FP32, m_type1: int = M_TYPE1) -> int:
    """Eq. 3."""
    return max(gamma_const(k, m_type3, m_type1), xi_const(m_type2, m_type1))


def slicing_feasible(rho: int, m_type1: int = M_TYPE1) -> bool:
    """The condition stated after Eq. 8, read at c = 0: floor(log2 sigma) = rho - 1, so it asks for
    m1 - (rho - 1) > 0, i.e. rho <= m1 (at least the sign digit survives in a slice)."""
    return m_type1 - (rho - 1) > 0


def table2_slice_count(k: int, m_type2: int, m_type3: int, m_type1: int = M_TYPE1):
    """Number of slices behind one cell of Table 2 (its entries are this number squared), or None
    where the table prints '--'.  Each slice advances by m1 - rho + 1 bits (b magnitude bits plus the
    sign digit gained by rounding to nearest), and the table counts ceil(m1 / (m1 - rho + 1))."""
    rho = rho_const(k, m_type2, m_type3, m_type1)
    if not slicing_feasible(rho, m_type1):
        return None
    per_slice = m_type1 - rho + 1
    return -(-m_type1 // per_slice)


@dataclass(frozen=True)
class Plan:
    fmt: str
    k: int
    k_block: int
    num_blocks: int
    rho: int
    b: int


def make_plan(k: int, fmt: str, k_block: int = 0) -> Plan:
    """rho from the block length (Section 4.3: the scheme is applied to each block, so Eq. 1 sees
    k_block, not k).  A short last block uses the same rho (safe: its k is smaller)."""
    kb = k if k_block in (0, None) else min(k_block, k)
    m2 = formats.SIGNIFICAND_BITS[fmt]
    m3 = formats.ACCUMULATOR_BITS[fmt]
    rho = rho_const(kb, m2, m3)
    # Eq. 1 assumes that a sum of magnitude 2^m3 is still exact, which holds for a floating-point accumulator; an INT32
    # accumulator ends at 2^31 - 1, so there one more bit goes to rho when k_block * 4^b would reach 2^31 exactly
    while kb << (2 * (M_TYPE1 - rho)) > formats.EXACT_WINDOW[fmt] and rho <= M_TYPE1:
        rho += 1
    if not slicing_feasible(rho):
        raise ValueError(f"slicing infeasible: rho={rho} for k_block={kb}, format {fmt}")
    nblk = -(-k // kb)
    return Plan(fmt=fmt, k=k, k_block=kb, num_blocks=nblk, rho=rho, b=M_TYPE1 - rho)


# --------------------------------------------------------------------------------------
# Eq. 4-8
# --------------------------------------------------------------------------------------
def ceil_log2_exact(mx: np.ndarray) -> np.ndarray:
    """Eq. 4 without libm rounding: smallest integer c with mx <= 2^c; 0 where mx == 0."""
    mant, e = np.frexp(mx)              # mx = mant * 2^e, mant in [0.5, 1)
    c = np.where(mant == 0.5, e - 1, e)
    return np.where(mx == 0, 0, c).astype(np.int64)


def slice_rows(X: np.ndarray, rho: int, num_slices: int):
    """Apply Eq. 4-8 to every row of X (rows are independent vectors x).

    Returns (slices, c, remainder): slices[p] is the real value of the Type2 slice (an array like X,
    entries q*2^(rho-53) with |q| <= 2^(53-rho)), c[p] the integer exponent vector of Eq. 4, and the
    remainder x^(s+1).
    """
    x = np.array(X, dtype=np.float64, copy=True)
    if not np.all(np.isfinite(x)):
        raise ValueError("non-finite input")
    slices, cs = [], []
    for _ in range(num_slices):
        mx = np.max(np.abs(x), axis=1) if x.shape[1] else np.zeros(x.shape[0])
        c = ceil_log2_exact(mx)                                  # Eq. 4
        sigma = np.ldexp(0.75, (rho + c).astype(np.int64))       # Eq. 5 (exact: a power-of-two multiple of 0.75)
        sig = sigma[:, None]
        v = (x + sig) - sig                                      # Eq. 6, two FP64 roundings, left to right
        x = x - v                                                # Eq. 7
        sl = np.ldexp(v, (-c)[:, None])                          # Eq. 8's scaling (exact)
        slices.append(sl)
        cs.append(c)
    return slices, cs, x


def slice_to_exhaustion(X: np.ndarray, rho: int, max_slices: int = 4096):
    """Eq. 4-8 repeated until the remainder vanishes (the stopping rule of the paragraph before Eq. 4): slices until
    every row's remainder is zero."""
    x = np.array(X, dtype=np.float64, copy=True)
    slices, cs = [], []
    while np.any(x != 0):
        if len(slices) >= max_slices:
            raise RuntimeError("slicing did not terminate")
        sl, c, x = slice_rows(x, rho, 1)
        slices.append(sl[0])
        cs.append(c[0])
    return slices, cs


def count_slices_to_exhaustion(X_rows: np.ndarray, fmt: str, k_block: int = 0) -> int:
    """Largest number of slices any block of any row of X_rows yields before its remainder is zero."""
    rows, k = X_rows.shape
    if rows == 0 or k == 0:
        return 0
    plan = make_plan(k, fmt, k_block)
    count = 0
    for t in range(plan.num_blocks):
        k0, k1 = t * plan.k_block, min(k, (t + 1) * plan.k_block)
        sl, _ = slice_to_exhaustion(X_rows[:, k0:k1], plan.rho)
        count = max(count, len(sl))
    return count


# --------------------------------------------------------------------------------------
# Eq. 10-11: slice-pair products
# --------------------------------------------------------------------------------------
def slice_integers(sl: np.ndarray, b: int) -> np.ndarray:
    """q = slice * 2^b as exact integers (float64 holding integers); checks |q| <= 2^b."""
    q = np.ldexp(sl, b)
    if not np.array_equal(q, np.rint(q)) or (q.size and np.max(np.abs(q)) > (1 << b)):
        raise AssertionError("slice entry is not an integer multiple of 2^-b within [-1, 1]")
    return q


def pair_product_int(qa: np.ndarray, qb: np.ndarray) -> np.ndarray:
    """Exact integer matrix of one slice pair: P[i, j] = sum_kk qa[i, kk] * qb[j, kk].
    The float64 matmul is exact here because every partial sum is an integer below 2^53."""
    P = qa @ qb.T
    Pi = P.astype(np.int64)
    assert np.array_equal(Pi.astype(np.float64), P)
    return Pi


def pair_order(num_slices: int, mode: str = "triangle") -> List[Tuple[int, int]]:
    """Slice pairs (p, q), 1-based, in accumulation order: anti-diagonals from the least significant
    (largest p+q) to the most significant, p ascending within one."""
    s = num_slices
    gmax = s + 1 if mode == "triangle" else 2 * s
    if mode not in ("triangle", "full"):
        raise ValueError(mode)
    order = []
    for g in range(gmax, 1, -1):
        for p in range(1, g):
            q = g - p
            if p <= s and q <= s:
                order.append((p, q))
    return order


# --------------------------------------------------------------------------------------
# FP64 accumulation (Section 3 after Eq. 11; Section 4.2 for the integer-emulated add)
# --------------------------------------------------------------------------------------
def hw_add(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    return x + y


@dataclass
class BlockResult:
    slices_a: List[np.ndarray]      # [p] -> (m, kb) real slice values
    slices_b: List[np.ndarray]      # [q] -> (n, kb)
    c_a: List[np.ndarray]           # [p] -> (m,) int
    c_b: List[np.ndarray]           # [q] -> (n,) int
    pairs: List[Tuple[int, int]]
    products: List[np.ndarray]      # per pair, exact int64 (m, n): sum of q_a*q_b; the FP32 value is this * 2^(-2b)
    S: np.ndarray                   # FP64 block sum


#: the accumulation rules of `block_result`
ACCUMULATE_RULES = ("plain", "runs", "exact")

#: "exact" rule: fraction bits of the fixed-point sum below the unit of the leading pair's product, 2^(c_x^(1)+c_y^(1)-2b)
EXACT_WINDOW_BITS = 144


def _accumulate_plain(terms, shape, add):
    """Eq. 10 as written, in Type1 = FP64 arithmetic: S = fl(S + 2^(c_x+c_y) * product), term after term."""
    S = np.zeros(shape, dtype=np.float64)
    for P, e in terms:
        S = add(S, np.ldexp(P.astype(np.float64), e))        # the term itself is exact: |P| <= 2^24, a power-of-two scale
    return S


def _accumulate_runs(terms, diagonals, shape, add):
    """Variant: consecutive terms of one anti-diagonal whose scale 2^(c_x+c_y) is the same for an element are
    summed exactly (integers in units of that scale), and each such run is added with one rounded FP64 addition.
    An exact sum does not depend on how it is formed, so a device is free to form it in the matrix unit's FP32
    accumulators (inside the window of Eq. 11) or in integer registers."""
    S = np.zeros(shape, dtype=np.float64)
    run_sum = np.zeros(shape, dtype=np.int64)          # exact sum of the current run, in units of 2^(run_e)
    run_e = np.zeros(shape, dtype=np.int64)
    open_run = np.zeros(shape, dtype=bool)
    run_diag = None                                    # anti-diagonal of the previous pair

    def flush(S, mask):
        term = np.where(mask, np.ldexp(run_sum.astype(np.float64), run_e), 0.0)   # exact: |run_sum| < 2^53
        return add(S, term)                                                        # adding +0.0 changes nothing

    for (P, e), g in zip(terms, diagonals):
        cont = open_run & (run_diag == g) & (e == run_e)   # a new anti-diagonal ends every run
        run_diag = g
        S = flush(S, open_run & ~cont)
        run_sum = np.where(cont, run_sum + P, P)
        run_e = e
        open_run = np.ones(shape, dtype=bool)
    return flush(S, open_run)


_to_float_rne = np.frompyfunc(float, 1, 1)             # Python's int -> float conversion rounds to nearest, ties to even


def _accumulate_exact(terms, e_lead, shape):
    """Variant: the sum of Eq. 10 carried out free of rounding error (remark after Eq. 11) as far as a fixed-point
    integer reaches, rounded to FP64 once.  Per element the unit is 2^(e_lead - EXACT_WINDOW_BITS), e_lead being the
    scale exponent of the leading pair (1,1); a term whose scale lies more than EXACT_WINDOW_BITS below e_lead is
    cut to that unit towards minus infinity (it is below 2^-128 of the leading product's unit), every other term
    is added exactly.  The order of the terms is irrelevant."""
    acc = np.zeros(shape, dtype=object)                # Python integers: no overflow, no rounding
    W = EXACT_WINDOW_BITS
    for P, e in terms:
        nz = P != 0
        sh = np.where(nz, W + (e - e_lead), 0)         # zero products (exhausted slices carry c = 0) add nothing
        Po = P.astype(object)
        up = np.left_shift(Po, np.maximum(sh, 0).astype(object))
        acc = acc + np.where(sh >= 0, up, np.right_shift(Po, np.maximum(-sh, 0).astype(object)))
    S = _to_float_rne(acc).astype(np.float64)
    return np.ldexp(S, e_lead - W)


def block_result(Ab: np.ndarray, Bb: np.ndarray, plan: Plan, num_slices: int, mode: str = "triangle",
                 add: Callable = hw_add, keep: bool = True, accumulate: str = "plain") -> BlockResult:
    """One k-block: slice rows of Ab (m x kb) and columns of Bb (kb x n), form the pair products, accumulate them
    element by element in `pair_order` with the rule `accumulate` ("plain" is the definition; see the module
    docstring and the three functions above)."""
    if accumulate not in ACCUMULATE_RULES:
        raise ValueError(accumulate)
    sa, ca, _ = slice_rows(Ab, plan.rho, num_slices)
    sb, cb, _ = slice_rows(np.ascontiguousarray(Bb.T), plan.rho, num_slices)
    qa = [slice_integers(s_, plan.b) for s_ in sa]
    qb = [slice_integers(s_, plan.b) for s_ in sb]
    limit = formats.EXACT_WINDOW[plan.fmt]
    shape = (Ab.shape[0], Bb.shape[1])
    pairs = pair_order(num_slices, mode)
    products, terms = [], []
    for (p, q) in pairs:
        P = pair_product_int(qa[p - 1], qb[q - 1])
        if P.size and np.max(np.abs(P)) > limit:
            raise AssertionError("pair product exceeds the exact range of the accumulator (Eq. 11 violated)")
        e = (ca[p - 1][:, None] + cb[q - 1][None, :] - 2 * plan.b).astype(np.int64)   # 2^(c_x+c_y) * 2^-2b
        terms.append((P, e))
        if keep:
            products.append(P)
    if accumulate == "plain":
        S = _accumulate_plain(terms, shape, add)
    elif accumulate == "runs":
        S = _accumulate_runs(terms, [p + q for p, q in pairs], shape, add)
    else:
        e_lead = (ca[0][:, None] + cb[0][None, :] - 2 * plan.b).astype(np.int64)
        S = _accumulate_exact(terms, e_lead, shape)
    return BlockResult(sa, sb, ca, cb, pairs, products, S)


def hw_mul(x, y):
    """FP64 multiplication of the host (IEEE, round to nearest even)."""
    return np.multiply(x, y, dtype=np.float64)


def ozaki_dgemm(A: np.ndarray, B: np.ndarray, fmt: str = "fp8", num_slices: int = 11, k_block: int = 0,
                mode: str = "triangle", add: Callable = hw_add, return_blocks: bool = False, accumulate: str = "plain",
                alpha: float = 1.0, beta: float = 0.0, C0: np.ndarray = None, mul: Callable = hw_mul):
    """C = A B by the Ozaki scheme with inner-product-wise blocking (Section 4.3): every block's sum is
    formed first (rule `accumulate`, see `block_result`), then added to C in FP64, blocks in ascending k.

    With alpha / beta (the GEMM of the BLAS the paper emulates, Section 1; the scaling needs the FP64
    multiplication that Section 4.2 emulates next to the addition) the product P formed as above is combined as
        C = fl(fl(alpha * P) + fl(beta * C0)),   beta == 0: C = fl(alpha * P) and C0 is not read,
        alpha == 1 and beta == 0: C = P (no arithmetic),
    one rounded multiplication per term and one rounded addition, no fused multiply-add."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    C = np.zeros((m, n), dtype=np.float64)
    blocks = []
    if k > 0:
        plan = make_plan(k, fmt, k_block)
        for t in range(plan.num_blocks):
            k0, k1 = t * plan.k_block, min(k, (t + 1) * plan.k_block)
            br = block_result(A[:, k0:k1], B[k0:k1, :], plan, num_slices, mode, add, keep=return_blocks, accumulate=accumulate)
            C = add(C, br.S)
            if return_blocks:
                blocks.append(br)
    if not (alpha == 1.0 and beta == 0.0):
        C = mul(np.float64(alpha), C)
        if beta != 0.0:
            C = add(C, mul(np.float64(beta), np.asarray(C0, dtype=np.float64)))
    return (C, blocks) if return_blocks else C


# --------------------------------------------------------------------------------------
# Type2 byte images of the slices (what the device must reproduce bit for bit)
# --------------------------------------------------------------------------------------
def split_operand(X_rows: np.ndarray, fmt: str, num_slices: int, k_block: int = 0):
    """Slice every row of X_rows (rows x k; for B pass B.T) block by block.

    Returns (codes, exps): codes[t][p] is the Type2 code array (rows x kb_t; uint8 for fp8, uint16 for
    fp16), exps[t][p] the int exponent vector.  The last block may be shorter."""
    rows, k = X_rows.shape
    plan = make_plan(k, fmt, k_block)
    codes, exps = [], []
    for t in range(plan.num_blocks):
        k0, k1 = t * plan.k_block, min(k, (t + 1) * plan.k_block)
        sl, cs, _ = slice_rows(X_rows[:, k0:k1], plan.rho, num_slices)
        codes.append([formats.encode_exact(fmt, s_, plan.b) for s_ in sl])
        exps.append([c.astype(np.int32) for c in cs])
    return codes, exps, plan
