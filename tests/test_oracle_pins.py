"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU needed).

Each test names the passage it pins.  None of them re-types the oracle's own formula:
they use values the paper prints (Table 2, Section 5.4), exact rational arithmetic,
the host FPU, an independent library conversion (torch's float8_e4m3fn) or closed forms.
"""
import dataclasses
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import exact, formats, ozaki_oracle as oz, softfloat
from paper_2508_00441_amd import inputs


# ------------------------------------------------------------------ Table 2 (Section 4.1)
def _read_table2(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "table2_min_gemms.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows.append((int(parts[0]), [None if p == "--" else int(p) for p in parts[1:]]))
    assert len(rows) == 16
    return rows


# columns of Table 2: (m_Type2, m_Type3)
_T2_COLUMNS = [(11, 24), (11, 11), (4, 24), (4, 11), (3, 24), (3, 11)]


def test_table2_all_cells_from_eq_1_to_3(golden_dir):
    for k, cells in _read_table2(golden_dir):
        for (m2, m3), printed in zip(_T2_COLUMNS, cells):
            s = oz.table2_slice_count(k, m2, m3)
            assert (None if s is None else s * s) == printed, (k, m2, m3)


@pytest.mark.parametrize("col", [0, 2, 4])
def test_table2_fp32_accumulate_columns_by_actually_slicing(golden_dir, col):
    """Slice full-mantissa one-binade vectors of length k until the remainder is zero and count."""
    m2, m3 = _T2_COLUMNS[col]
    rng = np.random.default_rng(7)
    for k, cells in _read_table2(golden_dir):
        rho = oz.rho_const(k, m2, m3)
        rows = 4 if k <= 16384 else 1
        X = inputs.full_mantissa_one_binade(rows, k, rng)
        X[:, ::2] *= -1.0
        sl, cs = oz.slice_to_exhaustion(X, rho)
        assert len(sl) ** 2 == cells[col], (k, len(sl))


def test_section_5_4_gemm_counts(golden_dir):
    want = {}
    with open(os.path.join(golden_dir, "kbk_gemm_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                kbk, g = line.split()
                want[int(kbk)] = int(g)
    assert want == {1024: 49, 4096: 64, 16384: 81}
    for kbk, g in want.items():
        assert oz.table2_slice_count(kbk, 11, 24) ** 2 == g
    # "121/81" at k = 8192
    assert oz.table2_slice_count(8192, 4, 24) ** 2 == 121 and oz.table2_slice_count(8192, 11, 24) ** 2 == 81


def test_gamma_matches_the_printed_formula_in_floating_point():
    for lk in range(0, 25):
        k = 1 << lk
        for m3 in (24, 11):
            assert oz.gamma_const(k, m3) == math.ceil(53 - (m3 - math.log2(k)) / 2)
    # between powers of two the integer form is the exact evaluation of the same expression
    for k in (3, 5, 1000, 1023, 1025, 5000, 65535, 65537, 100000):
        assert oz.gamma_const(k) == math.ceil(53 - (24 - math.log2(k)) / 2)


def test_plan_bits_per_slice():
    # largest b <= m2 with k_b * 4^b <= 2^24
    for k, b in [(16, 4), (8192, 4), (65536, 4), (65537, 3), (262144, 3), (262145, 2)]:
        assert oz.make_plan(k, "fp8").b == b
    for k, b in [(16, 10), (17, 9), (64, 9), (256, 8), (1024, 7), (4096, 6), (16384, 5), (65536, 4)]:
        assert oz.make_plan(k, "fp16").b == b
    p = oz.make_plan(16384, "fp16", 1024)
    assert (p.b, p.num_blocks, p.k_block) == (7, 16, 1024)
    p = oz.make_plan(1000, "fp8", 384)
    assert (p.num_blocks, p.k_block) == (3, 384)
    with pytest.raises(ValueError):
        oz.make_plan(1 << 25, "fp8")        # k * 4^0 > 2^24: not even one sign digit is exact


# ------------------------------------------------------------------ Eq. 4-9: the split is error-free
_nasty_rows = inputs.nasty_rows


@pytest.mark.parametrize("fmt,k", [("fp8", 64), ("fp16", 64), ("fp16", 1024), ("fp8", 4096), ("fp6", 64), ("fp6", 4096),
                                   ("fp6_e3m2", 64), ("fp6_e3m2", 4096), ("int8", 64), ("int8", 4096)])
def test_slices_sum_back_exactly_and_fit_their_format(fmt, k):
    rng = np.random.default_rng(11)
    X = _nasty_rows(rng, 12, k)
    plan = oz.make_plan(k, fmt)
    s = 9
    sl, cs, rem = oz.slice_rows(X, plan.rho, s)
    b = plan.b
    for p in range(s):
        q = np.ldexp(sl[p], b)
        assert np.array_equal(q, np.rint(q))                      # integer multiples of 2^-b
        assert np.max(np.abs(q)) <= 2 ** b                        # inside [-1, 1]
        codes = formats.encode_exact(fmt, sl[p], b)               # representable in Type2 ...
        assert np.array_equal(formats.decode(fmt, codes, b), sl[p])   # ... and round-trips
    # remainder after slice p is at most half an ulp of that slice
    sl1, cs1, rem1 = oz.slice_rows(X, plan.rho, 1)
    assert np.all(np.abs(rem1) <= np.ldexp(1.0, cs1[0] - b - 1)[:, None])
    # Eq. 9 in exact rational arithmetic, element by element (sampled columns to keep it quick)
    cols = rng.choice(k, size=min(k, 24), replace=False)
    for i in range(X.shape[0]):
        for j in cols:
            total = Fraction(float(rem[i, j]))
            for p in range(s):
                total += Fraction(float(sl[p][i, j])) * Fraction(2) ** int(cs[p][i])
            assert total == Fraction(float(X[i, j])), (i, j)


def test_exponent_rule_of_eq_4():
    mx = np.array([0.0, 1.0, np.nextafter(1.0, 2.0), np.nextafter(1.0, 0.0), 3.0, 4.0, 2.0 ** -1074, 0.75])
    assert list(oz.ceil_log2_exact(mx)) == [0, 0, 1, 0, 2, 2, -1074, 0]
    # away from powers of two the printed ceil(log2(.)) agrees
    rng = np.random.default_rng(3)
    v = np.exp(rng.normal(0, 20, 2000))
    frac = np.abs(np.log2(v) - np.rint(np.log2(v)))
    keep = frac > 1e-9
    assert np.array_equal(oz.ceil_log2_exact(v[keep]), np.ceil(np.log2(v[keep])).astype(np.int64))


def test_rounding_is_to_nearest_even_integer_multiple():
    """(x + sigma) - sigma must be x rounded to the nearest multiple of 2^(c-b), ties to even."""
    k = 64
    plan = oz.make_plan(k, "fp8")
    X = _nasty_rows(np.random.default_rng(5), 12, k)
    sl, cs, _ = oz.slice_rows(X, plan.rho, 1)
    for i in range(X.shape[0]):
        ulp = Fraction(2) ** int(cs[0][i] - plan.b)
        for j in range(k):
            t = Fraction(float(X[i, j])) / ulp
            fl = math.floor(t)
            diff = t - fl
            if diff > Fraction(1, 2) or (diff == Fraction(1, 2) and fl % 2 == 1):
                fl += 1
            assert Fraction(float(sl[0][i, j])) * Fraction(2) ** plan.b == fl, (i, j)


def test_e4m3_table_matches_torch_float8():
    torch = pytest.importorskip("torch")
    codes = np.arange(256, dtype=np.uint8)
    mine = formats.e4m3_decode(codes)
    theirs = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    both_nan = np.isnan(mine) & np.isnan(theirs)
    assert np.array_equal(mine[~both_nan], theirs[~both_nan]) and both_nan.sum() == 2
    # every slice value q/16 encodes to the byte torch produces
    vals = np.arange(-16, 17) / 16.0
    enc = formats.e4m3_encode_exact(vals)
    ref = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ref = np.where(vals == 0, 0, ref)
    assert np.array_equal(enc, ref)
    with pytest.raises(ValueError):
        formats.e4m3_encode_exact(np.array([17 / 16.0]))


def test_e2m3_table_has_the_published_format_constants():
    """OCP microscaling FP6 E2M3: bias 1, no infinities/NaNs, subnormals 0.125..0.875, normals 1.0..7.5."""
    vals = formats.e2m3_decode(np.arange(64, dtype=np.uint8))
    assert np.all(np.isfinite(vals))
    pos = vals[:32]
    assert np.array_equal(vals[32:], -pos)                                  # bit 5 is the sign
    assert np.all(np.diff(pos) > 0)                                         # codes ordered like their values
    assert pos[0] == 0.0 and pos[1] == 0.125 and pos[7] == 0.875            # subnormals: multiples of 1/8
    assert pos[8] == 1.0 and pos[31] == 7.5                                 # smallest / largest normal
    assert np.array_equal(pos[:16], np.arange(16) / 8.0)                    # step 1/8 up to 1.875
    assert np.array_equal(pos[16:24], 2.0 + np.arange(8) / 4.0) and np.array_equal(pos[24:], 4.0 + np.arange(8) / 2.0)
    # the 33 slice values q/16 are stored as q/8; q/16 itself is not representable for odd q
    sl = np.arange(-16, 17) / 16.0
    codes = formats.encode_exact("fp6", sl)
    assert codes.max() < 64 and np.array_equal(formats.decode("fp6", codes), sl)
    assert np.array_equal(formats.e2m3_decode(codes), 2.0 * sl)
    with pytest.raises(ValueError):
        formats.e2m3_encode_exact(np.array([1 / 16.0]))
    with pytest.raises(ValueError):
        formats.encode_exact("fp6", np.array([17 / 16.0]))


def test_e3m2_table_has_the_published_format_constants():
    """OCP microscaling FP6 E3M2 (Table 2's FP6 column): bias 3, no infinities/NaNs, subnormals 1/16 .. 3/16,
    normals 0.25 .. 28; three significand bits, so b = 3 and the slice values q/8 (|q| <= 8) are all codes."""
    vals = formats.e3m2_decode(np.arange(64, dtype=np.uint8))
    assert np.all(np.isfinite(vals))
    pos = vals[:32]
    assert np.array_equal(vals[32:], -pos) and np.all(np.diff(pos) > 0)
    assert pos[0] == 0.0 and pos[1] == 0.0625 and pos[3] == 0.1875 and pos[4] == 0.25 and pos[31] == 28.0
    assert oz.make_plan(4096, "fp6_e3m2").b == 3 and oz.make_plan(1 << 18, "fp6_e3m2").b == 3 and oz.make_plan(1 << 19, "fp6_e3m2").b == 2
    sl = np.arange(-8, 9) / 8.0
    codes = formats.encode_exact("fp6_e3m2", sl)
    assert codes.max() < 64 and np.array_equal(formats.decode("fp6_e3m2", codes), sl)
    with pytest.raises(ValueError):
        formats.encode_exact("fp6_e3m2", np.array([9 / 16.0]))          # needs four significand bits


def test_fp6_e2m3_has_the_slice_width_of_e4m3_and_gives_the_same_bits():
    """Four significand bits either way (Eq. 2), so plan, slices, exponents, products and C coincide."""
    for k, kb in ((8, 0), (4096, 0), (65536, 0), (262144, 0), (1000, 384)):
        assert oz.make_plan(k, "fp6", kb) == dataclasses.replace(oz.make_plan(k, "fp8", kb), fmt="fp6")
    assert oz.table2_slice_count(4096, formats.SIGNIFICAND_BITS["fp6"], 24) == 11          # the FP8 E4M3 column of Table 2
    rng = np.random.default_rng(66)
    A = inputs.phi_matrix(24, 200, 2.0, rng)
    B = inputs.phi_matrix(200, 20, 2.0, rng)
    for kb in (0, 64):
        C8, blk8 = oz.ozaki_dgemm(A, B, "fp8", 9, kb, return_blocks=True)
        C6, blk6 = oz.ozaki_dgemm(A, B, "fp6", 9, kb, return_blocks=True)
        assert np.array_equal(C8.view(np.uint64), C6.view(np.uint64))
        for b8, b6 in zip(blk8, blk6):
            assert all(np.array_equal(x, y) for x, y in zip(b8.products, b6.products))
    c8, e8, _ = oz.split_operand(A, "fp8", 9, 64)
    c6, e6, _ = oz.split_operand(A, "fp6", 9, 64)
    for t in range(len(c8)):
        for p in range(9):
            assert np.array_equal(formats.decode("fp8", c8[t][p]), formats.decode("fp6", c6[t][p]))
            assert np.array_equal(e8[t][p], e6[t][p])


# ------------------------------------------------------------------ Eq. 10-11
def _exact_sum_of_terms(blocks, b):
    """sum over blocks and pairs of 2^(cA+cB-2b) * P in exact rational arithmetic."""
    m, n = blocks[0].S.shape
    tot = [[Fraction(0) for _ in range(n)] for _ in range(m)]
    for br in blocks:
        for (p, q), P in zip(br.pairs, br.products):
            for i in range(m):
                for j in range(n):
                    if P[i, j]:
                        tot[i][j] += Fraction(int(P[i, j])) * Fraction(2) ** int(br.c_a[p - 1][i] + br.c_b[q - 1][j] - 2 * b)
    return tot


@pytest.mark.parametrize("fmt,kblock", [("fp8", 0), ("fp16", 0), ("fp8", 16), ("fp16", 10), ("fp6", 0), ("fp6", 16), ("fp6_e3m2", 0),
                                        ("int8", 0), ("int8", 16)])
def test_all_slices_all_pairs_equal_the_exact_product(fmt, kblock):
    """Eq. 10 with every slice and every pair is an identity: brute force on tiny, non-square inputs."""
    rng = np.random.default_rng(21)
    m, n, k = 5, 3, 37
    A = inputs.phi_matrix(m, k, 2.0, rng)
    B = inputs.phi_matrix(k, n, 2.0, rng)
    A[1, 4] = 0.0
    plan = oz.make_plan(k, fmt, kblock)
    s_full = 0
    for t in range(plan.num_blocks):
        k0, k1 = t * plan.k_block, min(k, (t + 1) * plan.k_block)
        s_full = max(s_full, len(oz.slice_to_exhaustion(A[:, k0:k1], plan.rho)[0]),
                     len(oz.slice_to_exhaustion(B[k0:k1, :].T.copy(), plan.rho)[0]))
    C, blocks = oz.ozaki_dgemm(A, B, fmt, s_full, kblock, mode="full", return_blocks=True)
    tot = _exact_sum_of_terms(blocks, plan.b)
    ref = exact.exact_matmul(A, B)
    for i in range(m):
        for j in range(n):
            assert tot[i][j] == ref[i][j], (i, j)
    # and the FP64-accumulated result is as good as a plain FP64 GEMM (Section 5.3)
    for i in range(m):
        for j in range(n):
            scale = exact.exact_dot(A[i, :], B[:, j], absolute=True)
            assert abs(Fraction(float(C[i, j])) - ref[i][j]) <= scale * Fraction(4 * k, 2 ** 53)


def test_pair_products_stay_inside_the_exact_fp32_window():
    """Eq. 11 at its edge: k = 65536 entries all equal to the row maximum -> q = 2^b everywhere."""
    k = 65536
    A = np.ones((2, k))
    B = np.ones((k, 2))
    B[:, 1] = -1.0
    C, blocks = oz.ozaki_dgemm(A, B, "fp8", 1, 0, return_blocks=True)
    P = blocks[0].products[0]
    assert np.array_equal(np.abs(P), np.full((2, 2), 1 << 24))
    assert np.array_equal(np.float32(P).astype(np.int64), P)       # representable in FP32
    assert np.array_equal(C, A @ B)
    # INT8 slices with INT32 accumulation: |q| <= 64, exact while k * 4^6 <= 2^31 - 1; one index more costs a slice bit
    assert oz.make_plan(524287, "int8").b == 6 and oz.make_plan(524288, "int8").b == 5
    k = 4096
    C, blocks = oz.ozaki_dgemm(np.ones((1, k)), -np.ones((k, 1)), "int8", 1, 0, return_blocks=True)
    assert int(blocks[0].products[0][0, 0]) == -k * 4096 and C[0, 0] == -k
    assert formats.int8_encode_exact(np.array([-1.0, 1.0, 0.5, -1 / 64]), 6).tolist() == [0xC0, 0x40, 0x20, 0xFF]
    with pytest.raises(ValueError):
        formats.int8_encode_exact(np.array([2.0]), 6)               # 128 does not fit a signed byte
    # k-blocking keeps FP16 slices inside the window as well
    k = 4096
    C, blocks = oz.ozaki_dgemm(np.ones((1, k)), np.ones((k, 1)), "fp16", 1, 1024, return_blocks=True)
    assert all(int(br.products[0][0, 0]) == 1 << 24 for br in blocks) and C[0, 0] == k


def test_integer_rows_need_one_slice_and_give_the_textbook_integer_product():
    rng = np.random.default_rng(2)
    m, n, k = 9, 7, 48
    QA = rng.integers(-16, 17, (m, k))
    QB = rng.integers(-16, 17, (k, n))
    QA[:, 0] = 16
    QB[0, :] = -16                                             # make every row/column maximum exactly 2^4
    ea = rng.integers(-30, 30, m)
    eb = rng.integers(-30, 30, n)
    A = np.ldexp(QA.astype(np.float64), ea[:, None])
    B = np.ldexp(QB.astype(np.float64), eb[None, :])
    C, blocks = oz.ozaki_dgemm(A, B, "fp8", 1, 0, return_blocks=True)
    assert np.array_equal(blocks[0].products[0], QA @ QB)
    assert np.array_equal(C, np.ldexp((QA @ QB).astype(np.float64), ea[:, None] + eb[None, :]))


def test_scaling_and_permutation_invariants():
    rng = np.random.default_rng(9)
    m, n, k = 6, 5, 40
    A = inputs.phi_matrix(m, k, 1.0, rng)
    B = inputs.phi_matrix(k, n, 1.0, rng)
    s = 6
    C, blk = oz.ozaki_dgemm(A, B, "fp8", s, 0, return_blocks=True)
    # scaling a row of A by 2^t shifts its exponents by t, leaves the slices alone, scales that row of C
    A2 = A.copy()
    A2[2, :] *= 2.0 ** 13
    C2, blk2 = oz.ozaki_dgemm(A2, B, "fp8", s, 0, return_blocks=True)
    for p in range(s):
        assert np.array_equal(blk2[0].slices_a[p], blk[0].slices_a[p])
        d = blk2[0].c_a[p] - blk[0].c_a[p]
        assert d[2] == 13 and np.all(np.delete(d, 2) == 0)
    C_expect = C.copy()
    C_expect[2, :] *= 2.0 ** 13
    assert np.array_equal(C2, C_expect)
    # permuting the inner index leaves every pair product and C unchanged
    perm = rng.permutation(k)
    C3, blk3 = oz.ozaki_dgemm(A[:, perm], B[perm, :], "fp8", s, 0, return_blocks=True)
    assert all(np.array_equal(x, y) for x, y in zip(blk3[0].products, blk[0].products))
    assert np.array_equal(C3, C)
    # (A B)^T = B^T A^T: transposed roles give the transposed pair products
    C4, blk4 = oz.ozaki_dgemm(B.T.copy(), A.T.copy(), "fp8", s, 0, return_blocks=True)
    pairs = blk[0].pairs
    for (p, q), P in zip(pairs, blk[0].products):
        P4 = blk4[0].products[blk4[0].pairs.index((q, p))]
        assert np.array_equal(P4, P.T)


def _read_hex_fixture(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, *vals = line.split()
                out[name] = np.array([float.fromhex(v) for v in vals])
    return out


def test_accumulation_rules_on_the_hand_derived_case(golden_dir):
    """Section 3 (after Eq. 11), Section 4 (order of accumulation): a 2 x 2 x 3 product worked with pencil and paper
    (tests/golden/accumulation_rules_2x2x3.txt) on which adding Eq. 10's terms one by one in FP64 (the definition,
    "plain") and adding equal-scale terms of an anti-diagonal exactly first ("runs") give different bits, and a
    1 x 1 x 3 product that sits on the cut of the fixed-point window of the "exact" rule."""
    g = _read_hex_fixture(os.path.join(golden_dir, "accumulation_rules_2x2x3.txt"))
    A, B = g["A"].reshape(2, 3), g["B"].reshape(3, 2)
    for rule in oz.ACCUMULATE_RULES:
        C = oz.ozaki_dgemm(A, B, "fp8", 3, 0, accumulate=rule)
        assert np.array_equal(C.view(np.uint64), g["C_" + rule].reshape(2, 2).view(np.uint64)), rule
        Csw = oz.ozaki_dgemm(A, B, "fp8", 3, 0, accumulate=rule, add=softfloat.soft_add)
        assert np.array_equal(Csw.view(np.uint64), C.view(np.uint64)), rule
    assert oz.ozaki_dgemm(A, B)[0, 0] != oz.ozaki_dgemm(A, B, accumulate="runs")[0, 0]      # the default is the plain rule
    # the fixture's own claim about the exact value, in rationals
    assert exact.exact_dot(A[0, :], B[:, 0]) == Fraction(1, 2 ** 14) + Fraction(1, 2 ** 62) == Fraction(float(g["C_runs"][0]))
    a2, b2 = g["a2"].reshape(1, 3), g["b2"].reshape(3, 1)
    for rule in oz.ACCUMULATE_RULES:
        assert oz.ozaki_dgemm(a2, b2, "fp8", 3, 0, accumulate=rule)[0, 0] == g["c2_" + rule][0], rule
    assert exact.round_fraction_to_double(exact.exact_dot(a2[0], b2[:, 0])) == g["c2_correctly_rounded"][0]


def test_exact_rule_with_all_slices_and_all_pairs_is_the_correctly_rounded_product():
    """Remark after Eq. 11: without rounding errors the sum of Eq. 10 IS the inner product.  With every slice, every
    pair and all scales inside the fixed-point window, the "exact" rule must therefore return the exact product
    (big-integer arithmetic of exact.py) rounded once; with k-blocking, the correctly rounded block products added
    in FP64."""
    rng = np.random.default_rng(77)
    m, n, k = 6, 5, 48
    A = inputs.phi_matrix(m, k, 1.5, rng)
    B = inputs.phi_matrix(k, n, 1.5, rng)
    A[2, :] = inputs.uniform_1_10(1, k, rng)[0]
    for fmt, kb in (("fp8", 0), ("fp16", 0), ("fp6_e3m2", 0), ("fp8", 16)):
        plan = oz.make_plan(k, fmt, kb)
        s_full = 0
        for t in range(plan.num_blocks):
            k0, k1 = t * plan.k_block, min(k, (t + 1) * plan.k_block)
            s_full = max(s_full, len(oz.slice_to_exhaustion(A[:, k0:k1], plan.rho)[0]),
                         len(oz.slice_to_exhaustion(B[k0:k1, :].T.copy(), plan.rho)[0]))
        C = oz.ozaki_dgemm(A, B, fmt, s_full, kb, mode="full", accumulate="exact")
        for i in range(m):
            for j in range(n):
                want = 0.0
                for t in range(plan.num_blocks):
                    k0, k1 = t * plan.k_block, min(k, (t + 1) * plan.k_block)
                    want = want + exact.round_fraction_to_double(exact.exact_dot(A[i, k0:k1], B[k0:k1, j]))
                assert C[i, j] == want, (fmt, kb, i, j)


def test_the_three_accumulation_rules_agree_within_rounding_and_runs_round_less_often():
    """The rules differ only in where FP64 roundings happen: on a regular exponent ladder (rows inside one binade)
    every anti-diagonal carries one scale, so "runs" performs one addition per anti-diagonal; all three stay within
    the bound of a plain FP64 GEMM of the exact product."""
    rng = np.random.default_rng(31)
    m, n, k = 4, 3, 64
    A = inputs.full_mantissa_one_binade(m, k, rng) * np.where(rng.random((m, k)) < 0.5, -1.0, 1.0)
    B = (inputs.full_mantissa_one_binade(n, k, rng) * np.where(rng.random((n, k)) < 0.5, -1.0, 1.0)).T.copy()
    ent = [(i, j) for i in range(m) for j in range(n)]
    for fmt, kb, s in (("fp8", 0, 7), ("fp16", 16, 4), ("fp8", 16, 6)):
        counts = {}
        for rule in ("plain", "runs"):
            calls = [0]

            def counting_add(x, y, calls=calls):
                calls[0] += int(np.count_nonzero(y[0, 0] if np.ndim(y) else y) > 0)
                return x + y
            oz.ozaki_dgemm(A[:1], B[:, :1], fmt, s, kb, accumulate=rule, add=counting_add)
            counts[rule] = calls[0]
        assert counts["runs"] < counts["plain"]
        errs = {}
        for rule in oz.ACCUMULATE_RULES:
            C = oz.ozaki_dgemm(A, B, fmt, s, kb, accumulate=rule)
            errs[rule] = exact.sampled_errors(A, B, ent, [C[i, j] for i, j in ent])[0]
        assert errs["exact"] <= errs["runs"] * 1.5 + 2.0 ** -60 and errs["runs"] <= errs["plain"] * 1.5 + 2.0 ** -60


def test_pair_order_is_least_significant_first():
    assert oz.pair_order(3) == [(1, 3), (2, 2), (3, 1), (1, 2), (2, 1), (1, 1)]
    assert len(oz.pair_order(16)) == 16 * 17 // 2
    full = oz.pair_order(3, "full")
    assert len(full) == 9 and full[0] == (3, 3) and full[-1] == (1, 1)


# ------------------------------------------------------------------ accuracy (Section 5.3)
def test_error_bound_and_decay_per_slice_on_the_small_config():
    m = n = k = 256
    A, B = inputs.phi_pair(m, n, k, 0.5, seed=0)
    ent = exact.sample_entries(m, n, 24, seed=5)
    rows = sorted({i for i, _ in ent})
    cols = sorted({j for _, j in ent})
    ri = {r: t for t, r in enumerate(rows)}
    ci = {c: t for t, c in enumerate(cols)}
    Asub, Bsub = A[rows, :], B[:, cols]
    errs = {}
    for s in (4, 6, 8, 10, 12):
        C = oz.ozaki_dgemm(Asub, Bsub, "fp8", s)
        errs[s] = exact.sampled_errors(A, B, ent, [C[ri[i], ci[j]] for i, j in ent])[0]
    bound = 4 * k * 2.0 ** -53
    assert errs[12] <= bound and errs[10] <= bound
    assert errs[4] > bound                                      # too few slices must show
    for s in (4, 6, 8):
        ratio = errs[s + 2] / errs[s]
        assert 2.0 ** -14 < ratio < 2.0 ** -6, (s, ratio)       # about 2^-(b+1) = 2^-5 per added slice
    native = exact.sampled_errors(A, B, ent, [(A @ B)[i, j] for i, j in ent])[0]
    assert errs[12] <= 4 * native + 2.0 ** -53


def test_k_blocking_stays_at_fp64_gemm_accuracy():
    m, n, k = 8, 8, 2048
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=3)
    ent = [(i, j) for i in range(m) for j in range(0, n, 3)]
    for fmt, kb, s in (("fp16", 256, 8), ("fp8", 512, 13), ("fp16", 1000, 9)):
        C = oz.ozaki_dgemm(A, B, fmt, s, kb)
        e_ab = exact.sampled_errors(A, B, ent, [C[i, j] for i, j in ent])[0]
        assert e_ab <= 4 * k * 2.0 ** -53


# ------------------------------------------------------------------ Section 4.2: integer-emulated FP64 add
def _random_normal_doubles(rng, n, emin=-300, emax=300):
    frac = rng.integers(0, 1 << 52, n, dtype=np.uint64)
    e = rng.integers(emin + 1023, emax + 1023, n, dtype=np.uint64)
    sign = rng.integers(0, 2, n, dtype=np.uint64)
    return ((sign << np.uint64(63)) | (e << np.uint64(52)) | frac).view(np.float64)


def test_soft_add_is_bitwise_the_host_fpu():
    rng = np.random.default_rng(2024)
    n = 2_000_000
    a = _random_normal_doubles(rng, 5 * n)
    parts = []
    # (1) unrelated operands, (2) exponent difference within +-70, (3) near-cancellation,
    # (4) exact ties: b = +-(odd multiple of) half an ulp of a, (5) equal exponents
    parts.append(_random_normal_doubles(rng, n))
    d = rng.integers(-70, 71, n)
    parts.append(np.ldexp(_random_normal_doubles(rng, n, -1, 1), np.frexp(a[n:2 * n])[1] + d))
    parts.append(-a[2 * n:3 * n] * (1.0 + np.ldexp(rng.integers(-8, 9, n).astype(np.float64), -rng.integers(30, 53, n))))
    ulp = np.ldexp(1.0, np.frexp(a[3 * n:4 * n])[1] - 53)
    parts.append(ulp * rng.choice([0.5, -0.5, 1.5, -1.5, 0.25, -0.25, 0.75], n))
    parts.append(np.copysign(np.ldexp(_random_normal_doubles(rng, n, -1, 1), np.frexp(a[4 * n:])[1]),
                             rng.choice([-1.0, 1.0], n)))
    b = np.concatenate(parts)
    assert a.size == b.size == 10_000_000
    got = softfloat.soft_add(a, b)
    want = a + b
    assert np.array_equal(got.view(np.uint64), want.view(np.uint64))
    # zeros
    z = np.array([0.0, -0.0, 0.0, -0.0, 1.5, 0.0, -2.5])
    w = np.array([0.0, 0.0, -0.0, -0.0, 0.0, -3.0, 2.5])
    assert np.array_equal(softfloat.soft_add(z, w).view(np.uint64), (z + w).view(np.uint64))


def test_emulated_accumulation_gives_the_same_bits():
    A, B = inputs.phi_pair(24, 20, 96, 2.0, seed=4)
    for fmt, kb in (("fp8", 0), ("fp16", 32)):
        C_hw = oz.ozaki_dgemm(A, B, fmt, 9, kb)
        C_sw = oz.ozaki_dgemm(A, B, fmt, 9, kb, add=softfloat.soft_add)
        assert np.array_equal(C_hw.view(np.uint64), C_sw.view(np.uint64))


def test_soft_mul_is_bitwise_the_host_fpu():
    """Section 4.2: the integer-only multiplication equals the hardware one bit for bit (normal range)."""
    rng = np.random.default_rng(23)
    n = 2_000_000

    def rnd(cnt, lo, hi):
        frac = rng.integers(0, 1 << 52, cnt, dtype=np.uint64)
        e = rng.integers(lo + 1023, hi + 1023, cnt, dtype=np.uint64)
        sg = rng.integers(0, 2, cnt, dtype=np.uint64)
        return ((sg << np.uint64(63)) | (e << np.uint64(52)) | frac).view(np.float64)

    a = rnd(5 * n, -300, 300)
    b = rnd(5 * n, -300, 300)
    # products that are exactly representable or exact ties: few significant bits in both factors
    a[n:2 * n] = np.ldexp(rng.integers(1, 1 << 27, n).astype(np.float64), rng.integers(-200, 200, n))
    b[n:2 * n] = np.ldexp(rng.integers(1, 1 << 27, n).astype(np.float64), rng.integers(-200, 200, n))
    # significands whose product lands next to a power of two (rounding carries into the next binade)
    a[2 * n:3 * n] = np.nextafter(2.0, 0.0) * np.ldexp(1.0, rng.integers(-100, 100, n))
    b[2 * n:3 * n] = (1.0 + np.ldexp(rng.integers(0, 8, n).astype(np.float64), -52)) * np.ldexp(1.0, rng.integers(-100, 100, n))
    a[:4] = [0.0, -0.0, 3.0, -1.5]
    b[:4] = [5.0, 2.0, 0.0, -0.0]
    got = softfloat.soft_mul(a, b)
    assert np.array_equal(got.view(np.uint64), (a * b).view(np.uint64))
    # the bit-level entry point and one value worked by hand: (1 + 2^-52)^2 = 1 + 2^-51 + 2^-104 -> 1 + 2^-51
    x = np.nextafter(1.0, 2.0)
    assert softfloat.soft_mul_bits(int(np.float64(x).view(np.uint64)), int(np.float64(x).view(np.uint64))) == int(np.float64(1.0 + 2.0 ** -51).view(np.uint64))


def test_alpha_beta_combination_follows_its_definition():
    """C = fl(fl(alpha P) + fl(beta C0)) around the product P of the plain call; emulated arithmetic gives the same bits."""
    rng = np.random.default_rng(31)
    A = inputs.phi_matrix(20, 96, 1.0, rng)
    B = inputs.phi_matrix(96, 24, 1.0, rng)
    C0 = inputs.phi_matrix(20, 24, 2.0, rng)
    P = oz.ozaki_dgemm(A, B, "fp8", 9, 32)
    for alpha, beta in ((1.0, 0.0), (-2.5, 0.0), (1.0, 1.0), (0.3, -1.7), (0.0, 2.0)):
        C = oz.ozaki_dgemm(A, B, "fp8", 9, 32, alpha=alpha, beta=beta, C0=C0)
        want = P if (alpha, beta) == (1.0, 0.0) else (alpha * P if beta == 0.0 else alpha * P + beta * C0)
        assert np.array_equal(C.view(np.uint64), want.view(np.uint64)), (alpha, beta)
        Csw = oz.ozaki_dgemm(A, B, "fp8", 9, 32, alpha=alpha, beta=beta, C0=C0, add=softfloat.soft_add, mul=softfloat.soft_mul)
        assert np.array_equal(C.view(np.uint64), Csw.view(np.uint64)), (alpha, beta)
    # beta == 0 does not read C0 (BLAS convention): NaNs there do not propagate
    Cn = oz.ozaki_dgemm(A, B, "fp8", 9, 32, alpha=2.0, beta=0.0, C0=np.full((20, 24), np.nan))
    assert np.array_equal(Cn, 2.0 * P)
    # against the exact product: alpha * (A B) + beta * C0 within the GEMM bound plus the three extra roundings
    ent = exact.sample_entries(20, 24, 12, seed=3)
    C = oz.ozaki_dgemm(A, B, "fp8", 11, 32, alpha=0.3, beta=-1.7, C0=C0)
    for i, j in ent:
        ex = Fraction(0.3) * exact.exact_dot(A[i, :], B[:, j]) + Fraction(-1.7) * Fraction(float(C0[i, j]))
        scale = abs(0.3) * float(np.abs(A[i, :]) @ np.abs(B[:, j])) + 1.7 * abs(float(C0[i, j]))
        assert abs(Fraction(float(C[i, j])) - ex) <= Fraction(4 * 96 * 2.0 ** -53 + 3 * 2.0 ** -53) * Fraction(scale)


def test_exact_reference_is_exact():
    # closed form: sum_{i<=N} i*(N+1-i) = N(N+1)(N+2)/6, with a huge cancelling pair on top
    N = 500
    x = np.arange(1, N + 1, dtype=np.float64)
    y = x[::-1].copy()
    assert exact.exact_dot(x, y) == Fraction(N * (N + 1) * (N + 2), 6)
    x2 = np.concatenate([x, [2.0 ** 600, -(2.0 ** 600)]])
    y2 = np.concatenate([y, [2.0 ** 300, 2.0 ** 300]])
    assert exact.exact_dot(x2, y2) == Fraction(N * (N + 1) * (N + 2), 6)
    assert exact.exact_dot(np.array([0.1]), np.array([0.1])) == Fraction(0.1) * Fraction(0.1)
    assert exact.exact_dot(np.array([-0.1, 3.0]), np.array([0.1, 1.0]), absolute=True) == Fraction(0.1) * Fraction(0.1) + 3


def test_fast_exact_residuals_agree_with_big_integers():
    """exact.dot_residuals (halves of 26 bits, math.fsum) against the big-integer exact_dot: the residual c_hat - x.y
    and the product itself, both rounded once, on wide-range, cancelling and benchmark-like vectors."""
    rng = np.random.default_rng(404)
    cases = []
    for phi, k in ((0.5, 300), (4.0, 1000), (2.0, 4096)):
        cases.append((inputs.phi_matrix(1, k, phi, rng)[0], inputs.phi_matrix(1, k, phi, rng)[0]))
    x = inputs.full_mantissa_one_binade(1, 512, rng)[0]
    cases.append((np.concatenate([x, -x]), np.concatenate([x[::-1], x[::-1]]) * (1 + 2.0 ** -30)))      # heavy cancellation
    cases.append((np.array([2.0 ** 500, 1.0, -(2.0 ** 500)]), np.array([2.0 ** 300, 3.0, 2.0 ** 300])))
    for x, y in cases:
        ex = exact.exact_dot(x, y)
        for c_hat in (float(x @ y), exact.round_fraction_to_double(ex), 0.0, 1.25 * float(x @ y) + 1e-300):
            res, dot = exact.dot_residuals(x, y, c_hat)
            assert res == exact.round_fraction_to_double(Fraction(c_hat) - ex)
            assert dot == exact.round_fraction_to_double(ex)
    A, B = inputs.phi_pair(6, 5, 700, 3.0, seed=8)
    ent = [(i, j) for i in range(6) for j in range(5)]
    C = A @ B
    slow = exact.sampled_errors(A, B, ent, [C[i, j] for i, j in ent])
    fast = exact.sampled_errors_fast(A, B, ent, [C[i, j] for i, j in ent])
    assert np.allclose(slow[2], fast[2], rtol=1e-9, atol=0) and np.allclose(slow[3], fast[3], rtol=1e-9, atol=0)
    # distance in units in the last place
    a = np.array([1.0, 1.0, -0.0, -1.0, 2.0 ** -1074])
    b = np.array([np.nextafter(1.0, 2.0), np.nextafter(np.nextafter(1.0, 0.0), 0.0), 0.0, 1.0, -(2.0 ** -1074)])
    assert list(exact.ulp_distance(a, b)) == [1, 2, 0, 2 * 0x3FF0000000000000, 2]
