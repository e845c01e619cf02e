"""Host-side checks of the product that need no GPU: the C-ABI library loads and exports every symbol the
header declares, the host planner agrees with the oracle's constants, and the integer-only FP64 routines
(compiled for the host) agree with the host FPU."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import ozaki_oracle as oz
from paper_2508_00441_amd import binding as lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(lib.LIB_PATH):
        from paper_2508_00441_amd import build
        build.build_library(verbose=False)
    lib.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "ozaki_dgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ozaki_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 14
    raw = ctypes.CDLL(lib.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), name
    assert sorted(lib.SIGNATURES) == names           # the binding covers the same set, no more, no less


def test_planner_matches_eq_1_to_3():
    for fmt, fid in (("fp8", lib.SLICE_FP8_E4M3), ("fp16", lib.SLICE_FP16), ("fp6", lib.SLICE_FP6_E2M3), ("fp6_e3m2", lib.SLICE_FP6_E3M2),
                     ("int8", lib.SLICE_INT8)):
        for k in [1, 2, 3, 8, 16, 17, 64, 65, 255, 256, 1024, 1025, 4096, 5000, 16384, 16385, 65536, 65537, 262144, 524287, 524288,
                  1 << 24]:
            p = oz.make_plan(k, fmt)
            assert lib.ozaki_plan(k, fid) == (p.rho, p.b), (fmt, k)
    with pytest.raises(lib.OzakiError) as e:
        lib.ozaki_plan((1 << 24) + 1, lib.SLICE_FP8_E4M3)
    assert e.value.status == lib.STATUS_INFEASIBLE
    assert lib.ozaki_plan((1 << 31) - 1, lib.SLICE_INT8) == (53, 0)
    with pytest.raises(lib.OzakiError) as e:
        lib.ozaki_plan(1 << 31, lib.SLICE_INT8)
    assert e.value.status == lib.STATUS_INFEASIBLE
    with pytest.raises(lib.OzakiError) as e:
        lib.ozaki_plan(0, 0)
    assert e.value.status == -1
    with pytest.raises(lib.OzakiError) as e:
        lib.ozaki_plan(16, 7)
    assert e.value.status == -2


def test_k_block_suggestion_keeps_the_plan_feasible():
    """A heuristic (parity unpinned); what is checked: the suggested block is accepted by the planner."""
    for fid in (lib.SLICE_FP8_E4M3, lib.SLICE_FP16, lib.SLICE_FP6_E2M3, lib.SLICE_FP6_E3M2, lib.SLICE_INT8):
        for k in (1, 100, 4096, 4097, 16384, 32768, 32769, 65536, 65537, 1 << 20, 1 << 26):
            kb = lib.ozaki_suggest_k_block(k, fid)
            assert 0 <= kb <= k
            assert lib.ozaki_workspace_bytes(64, 64, k, fid, 4, kb) > 0
            assert lib.ozaki_plan(kb or k, fid)[1] >= 3                        # the suggestion keeps the slices wide
    assert lib.ozaki_suggest_k_block(16384, lib.SLICE_FP16) == 4096 and lib.ozaki_suggest_k_block(16384, lib.SLICE_FP8_E4M3) == 0
    with pytest.raises(lib.OzakiError):
        lib.ozaki_suggest_k_block(16, 9)


def test_workspace_sizes():
    full = lib.ozaki_workspace_bytes(8192, 8192, 8192, 0, 16, 0)
    mini = lib.ozaki_workspace_min_bytes(8192, 8192, 8192, 0, 16, 0)
    pair = 8192 * 8192 * 4
    slices = 2 * 16 * 8192 * 8192
    assert full >= 136 * pair + slices + 8192 * 8192 * 8
    assert slices + 8192 * 8192 * 8 + pair < mini < full
    # more pairs than the resident-product budget: capped, with room for the running block sum (three 64-bit words)
    big = lib.ozaki_workspace_bytes(32768, 32768, 16384, 0, 13, 0)          # 91 products of 4 GiB
    assert big < (160 << 30) + 2 * 13 * 32768 * 16384 + 32768 * 16384 * 8 + 3 * 32768 * 32768 * 8 + (16 << 20)   # + A transposed + three sum words
    assert lib.ozaki_workspace_bytes(16, 16, 16, 5, 4, 0) == 0          # bad format
    assert lib.ozaki_workspace_bytes(16, 16, 1 << 25, 0, 4, 0) == 0     # no slice width is exact for a block this long
    assert lib.ozaki_workspace_bytes(16, 16, 1 << 25, 0, 4, 8192) > 0
    # blocks beyond the register-resident slicing kernel need its streaming state: 12 bytes per (padded) element
    long_ws = lib.ozaki_workspace_bytes(16, 16, 1 << 20, 0, 4, 0)
    assert long_ws > lib.ozaki_workspace_bytes(16, 16, 1 << 20, 0, 4, 16384) + 12 * 32 * (1 << 20) - (1 << 20)
    assert lib.ozaki_workspace_bytes(16, 16, 16, 0, 33, 0) == 0         # more slices than the library takes
    assert lib.ozaki_workspace_bytes(0, 0, 0, 0, 4, 0) >= 256
    tri = lib.ozaki_workspace_bytes(1024, 1024, 1024, 0, 8, 0)
    allp = lib.ozaki_workspace_bytes_ex(1024, 1024, 1024, 0, 8, 0, lib.PAIRS_ALL, 0)
    assert allp - tri == (64 - 36) * 1024 * 1024 * 4                   # s*s instead of s(s+1)/2 products
    assert lib.ozaki_workspace_bytes_ex(1024, 1024, 1024, 0, 8, 0, lib.PAIRS_TRIANGLE, 1) == lib.ozaki_workspace_min_bytes(1024, 1024, 1024, 0, 8, 0)
    assert lib.ozaki_workspace_bytes_ex(1024, 1024, 1024, 0, 8, 0, 2, 0) == 0


def test_argument_errors_are_reported_before_anything_is_launched():
    f = lib.load().ozaki_dgemm
    assert f(-1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 0) == -1
    assert f(1, -1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 0) == -2
    assert f(1, 1, -1, None, 1, None, 1, None, 1, 0, 4, 0, 0) == -3
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 9, 4, 0, 0) == -10
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 0, -4, 0, 0) == -11
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, -1, 0) == -12
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 5) == -13
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, -1) == -13
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 0) == -8       # C missing
    assert f(1, 1, 1, None, 1, None, 1, 1 << 20, 1, 0, 4, 0, 0) == -4    # A missing
    assert f(1, 1, 1 << 25, None, 1, None, 1, None, 1, 0, 4, 0, 0) == lib.STATUS_INFEASIBLE
    assert f(1, 1, 1 << 25, None, 1, None, 1, None, 1, 0, 4, 4096, 0) == -8             # blocked: feasible, C missing
    assert f(1, 1, 1, None, 1, None, 1, None, 1, 0, 33, 0, 0) == lib.STATUS_SLICE_COUNT
    assert len({lib.status_string(c) for c in (1, 3, 4, 5, 6, 7)}) == 6                  # every cause has a message of its own
    fx = lib.load().ozaki_dgemm_ex
    assert fx(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 0, 5, 0, 0) == -14
    assert fx(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 0, 1, 7, 0) == -15
    assert fx(1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 2, 1, 1, 0) == -8             # exact mode, all pairs: C missing
    fs = lib.load().ozaki_dgemm_static
    assert fs(-1, 1, 1, None, 1, None, 1, None, 1, 0, 4, 0, 0) == -1
    assert fs(4096, 4096, 4096, 1 << 20, 4096, 1 << 20, 4096, 1 << 20, 4096, 0, 13, 0, 0) == lib.STATUS_STATIC_LIMIT
    assert f(0, 0, 5, None, 1, None, 1, None, 1, 0, 4, 0, 0) == 0        # empty product: nothing to do
    assert "workspace" in lib.status_string(lib.STATUS_WORKSPACE)
    assert "argument" in lib.status_string(-3)
    # the scaled call counts positions in its own argument list (alpha is 4th, beta 9th)
    g = lib.load().ozaki_dgemm_scaled
    assert g(1, 1, -1, 2.0, None, 1, None, 1, 0.5, None, 1, 0, 4, 0, 0) == -3
    assert g(1, 1, 1, float("inf"), None, 1, None, 1, 0.5, None, 1, 0, 4, 0, 0) == -4
    assert g(1, 1, 1, 2.0, None, 1, None, 1, float("nan"), None, 1, 0, 4, 0, 0) == -9
    assert g(1, 1, 1, 2.0, None, 1, None, 1, 5e-324, None, 1, 0, 4, 0, 0) == -9          # subnormal scalar
    assert g(1, 1, 1, 2.0, None, 1, None, 1, 0.5, None, 1, 0, 4, 0, 0) == -10             # C missing
    assert g(1, 1, 1, 2.0, None, 1, None, 1, 0.5, 1 << 20, 1, 0, 4, 0, 0) == -5           # A missing
    assert g(1, 1, 1, 2.0, None, 1, None, 1, 0.5, None, 1, 9, 4, 0, 0) == -12             # bad format
    assert g(1, 1, 1, 2.0, None, 1, None, 1, 0.5, None, 1, 0, 4, 0, 5) == -15             # bad accumulation mode
    assert g(1, 1, 1, 2.0, 1 << 20, 1, 1 << 20, 1, 0.5, 1 << 20, 1, 0, 4, 0, 0) == lib.STATUS_WORKSPACE
    assert lib.ozaki_workspace_bytes_scaled(1000, 500, 64, 0, 4, 0) - lib.ozaki_workspace_bytes(1000, 500, 64, 0, 4, 0) == 1000 * 500 * 8


@pytest.fixture(scope="module")
def host_emu(tmp_path_factory):
    out = tmp_path_factory.mktemp("emu") / "libhostemu.so"
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", str(out),
                           os.path.join(ROOT, "tests", "host_fp64_emu_harness.cpp")])
    return ctypes.CDLL(str(out))


def _rnd(rng, n, lo, hi):
    frac = rng.integers(0, 1 << 52, n, dtype=np.uint64)
    e = rng.integers(lo + 1023, hi + 1023, n, dtype=np.uint64)
    sg = rng.integers(0, 2, n, dtype=np.uint64)
    return ((sg << np.uint64(63)) | (e << np.uint64(52)) | frac).view(np.float64)


def test_product_fp64_add_emulation_on_host_equals_fpu(host_emu):
    rng = np.random.default_rng(5)
    n = 1_000_000
    a = _rnd(rng, 4 * n, -300, 300)
    ulp = np.ldexp(1.0, np.frexp(a[3 * n:])[1] - 53)
    b = np.concatenate([
        _rnd(rng, n, -300, 300),
        np.ldexp(_rnd(rng, n, -1, 1), np.frexp(a[n:2 * n])[1] + rng.integers(-70, 71, n)),
        -a[2 * n:3 * n] * (1.0 + np.ldexp(rng.integers(-8, 9, n).astype(np.float64), -rng.integers(30, 53, n))),
        ulp * rng.choice([0.5, -0.5, 1.5, -1.5, 0.25, -0.25, 0.75], n),
    ])
    a[:5] = [0.0, -0.0, 1.5, 0.0, -2.5]
    b[:5] = [-0.0, -0.0, 0.0, -3.0, 2.5]
    out = np.empty_like(a)
    host_emu.host_fp64_add_emulated(a.ctypes.data_as(ctypes.c_void_p), b.ctypes.data_as(ctypes.c_void_p),
                                    out.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(a.size))
    assert np.array_equal(out.view(np.uint64), (a + b).view(np.uint64))


def test_product_fp64_mul_emulation_on_host_equals_fpu(host_emu):
    rng = np.random.default_rng(9)
    n = 1_000_000
    a = _rnd(rng, 4 * n, -300, 300)
    b = _rnd(rng, 4 * n, -300, 300)
    # short significands: exact products and exact ties
    a[n:2 * n] = np.ldexp(rng.integers(1, 1 << 27, n).astype(np.float64), rng.integers(-200, 200, n))
    b[n:2 * n] = np.ldexp(rng.integers(1, 1 << 27, n).astype(np.float64), rng.integers(-200, 200, n))
    # products next to a power of two
    a[2 * n:3 * n] = np.nextafter(2.0, 0.0) * np.ldexp(1.0, rng.integers(-100, 100, n))
    b[2 * n:3 * n] = (1.0 + np.ldexp(rng.integers(0, 8, n).astype(np.float64), -52)) * np.ldexp(1.0, rng.integers(-100, 100, n))
    a[:4] = [0.0, -0.0, 3.0, -1.5]
    b[:4] = [5.0, 2.0, 0.0, -0.0]
    out = np.empty_like(a)
    host_emu.host_fp64_mul_emulated(a.ctypes.data_as(ctypes.c_void_p), b.ctypes.data_as(ctypes.c_void_p),
                                    out.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(a.size))
    assert np.array_equal(out.view(np.uint64), (a * b).view(np.uint64))
    # the 128-bit product against Python integers (Section 4.2's four partial products)
    x = rng.integers(0, 1 << 63, 20000, dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, 20000, dtype=np.uint64)
    y = rng.integers(0, 1 << 63, 20000, dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, 20000, dtype=np.uint64)
    x[:3] = [0, 2 ** 64 - 1, 2 ** 64 - 1]
    y[:3] = [5, 2 ** 64 - 1, 1]
    hi = np.empty_like(x)
    lo = np.empty_like(x)
    host_emu.host_mul_64x64_128(x.ctypes.data_as(ctypes.c_void_p), y.ctypes.data_as(ctypes.c_void_p),
                                hi.ctypes.data_as(ctypes.c_void_p), lo.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(x.size))
    for xi, yi, h, l in zip(x.tolist(), y.tolist(), hi.tolist(), lo.tolist()):
        assert (h << 64) | l == xi * yi


def test_product_power_of_two_scaling_on_host(host_emu):
    rng = np.random.default_rng(6)
    n = 500_000
    f = np.ldexp(rng.integers(-(1 << 24), (1 << 24) + 1, n).astype(np.float64), -8)
    x = np.ldexp(f, rng.integers(-300, 300, n))
    e2 = rng.integers(-300, 300, n).astype(np.int32)
    out = np.empty(n, dtype=np.uint64)
    host_emu.host_fp64_scale_pow2(x.ctypes.data_as(ctypes.c_void_p), e2.ctypes.data_as(ctypes.c_void_p),
                                  out.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(n))
    assert np.array_equal(out, np.ldexp(x, e2).view(np.uint64))


def test_product_integer_conversions_on_host(host_emu):
    rng = np.random.default_rng(8)
    n = 400_000
    bits = rng.integers(1, 54, n)                                   # all magnitudes below 2^53, every bit length
    v = (rng.integers(0, 1 << 53, n) >> (53 - bits)) * rng.choice([-1, 1], n)
    v[:6] = [0, 1, -1, (1 << 31) - 1, (1 << 53) - 1, -(1 << 53) + 1]
    v = v.astype(np.int64)
    e2 = rng.integers(-300, 300, n).astype(np.int32)
    out = np.empty(n, dtype=np.uint64)
    host_emu.host_int53_scaled_to_fp64(v.ctypes.data_as(ctypes.c_void_p), e2.ctypes.data_as(ctypes.c_void_p),
                                       out.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(n))
    want = np.ldexp(v.astype(np.float64), e2)
    assert np.array_equal(out, want.view(np.uint64))



def test_product_rounded_sum_on_host_equals_chain_of_fpu_additions(host_emu):
    """The accumulation kernel's running sum (an integer addition and one rounding to 53 bits where both operands fit
    64 bits, the general emulated addition elsewhere) must give the bits of the plain chain of rounded FP64 additions, for the exponent patterns the method produces
    (terms about 2^b apart, least significant first) and for arbitrary ones (cancellation, reordering, ties)."""
    rng = np.random.default_rng(12)
    n_seq, length = 60_000, 18
    v = rng.integers(-(1 << 29), (1 << 29) + 1, (n_seq, length)).astype(np.int64)
    v[::5] *= 1 << 8                                                                           # sums of INT32 products: up to 2^37
    v[rng.random((n_seq, length)) < 0.1] = 0
    small = rng.random((n_seq, length)) < 0.3
    v[small] = rng.integers(-40, 41, int(small.sum()))
    e2 = np.empty((n_seq, length), dtype=np.int32)
    third = n_seq // 3
    e2[:third] = -100 + np.cumsum(rng.integers(3, 7, (third, length)), axis=1)                 # ascending, like anti-diagonals
    e2[third:2 * third] = rng.integers(-60, 60, (third, length))                              # unordered
    e2[2 * third:] = rng.integers(-3, 4, (n_seq - 2 * third, length))                         # close: long stretches without any rounding
    v[2 * third:2 * third + 2000, 1] = -v[2 * third:2 * third + 2000, 0]                      # exact cancellation ...
    e2[2 * third:2 * third + 2000, 1] = e2[2 * third:2 * third + 2000, 0]                     # ... back to zero
    # a sum that rounds up to a power of two (2^54 - 1 -> 2^54: the integer significand reaches 2^53) and goes on
    v[1], e2[1] = 0, 0
    v[1, :4], e2[1, :4] = [(1 << 52) - 1, 3, 1, -5], [2, 0, 0, 1]
    # the same with the signs turned, and a sum that hits a negative power of two exactly (-2^53, then 1 is added twice)
    v[2], e2[2] = 0, 0
    v[2, :4], e2[2, :4] = [-((1 << 52) - 1), -3, -1, 5], [2, 0, 0, 1]
    v[4], e2[4] = 0, 0
    v[4, :4], e2[4, :4] = [-(1 << 51), -(1 << 51), 1, 1], [1, 1, 0, 0]
    start = np.zeros(n_seq, dtype=np.float64)
    start[::7] = _rnd(rng, start[::7].size, -40, 40)                                          # continued block sums
    out = np.empty(n_seq, dtype=np.uint64)
    exact_adds = ctypes.c_longlong(0)
    v, e2 = np.ascontiguousarray(v), np.ascontiguousarray(e2)
    host_emu.host_rounded_sum(v.ctypes.data_as(ctypes.c_void_p), e2.ctypes.data_as(ctypes.c_void_p), start.ctypes.data_as(ctypes.c_void_p),
                              out.ctypes.data_as(ctypes.c_void_p), ctypes.byref(exact_adds), ctypes.c_size_t(n_seq), ctypes.c_size_t(length))
    want = start.copy()
    for j in range(length):
        want = want + np.ldexp(v[:, j].astype(np.float64), e2[:, j])
    assert np.array_equal(out, want.view(np.uint64))
    # both routes are exercised: most additions on integers, a good number through the general routine
    share = exact_adds.value / (n_seq * length)
    print("share of integer additions", share)
    assert 0.5 < share < 0.98


def test_product_fixed_point_accumulator_on_host_equals_python_integers(host_emu):
    """The exact accumulation mode's 192-bit sum and its single rounding against Python's unbounded integers and its
    correctly rounded int -> float conversion: random terms over the whole window, terms below the unit (cut towards
    minus infinity), cancellation down to a few bits, exact ties."""
    rng = np.random.default_rng(44)
    n_seq, length = 40_000, 24
    v = rng.integers(-(1 << 36), (1 << 36) + 1, (n_seq, length)).astype(np.int64)
    small = rng.random((n_seq, length)) < 0.4
    v[small] = rng.integers(-(1 << 24), (1 << 24) + 1, int(small.sum()))
    v[rng.random((n_seq, length)) < 0.1] = 0
    sh = rng.integers(-80, 145, (n_seq, length)).astype(np.int32)
    q = n_seq // 4
    sh[:q] = np.minimum(144, np.cumsum(rng.integers(0, 9, (q, length)), axis=1))               # ascending ladders from the unit
    sh[q:2 * q] = rng.integers(0, 3, (q, length))                                              # short sums: the exact branch
    v[2 * q:2 * q + 3000, 1] = -v[2 * q:2 * q + 3000, 0]                                       # cancellation of the two
    sh[2 * q:2 * q + 3000, 1] = sh[2 * q:2 * q + 3000, 0]                                      # largest terms
    # exact ties: 2^60 + 2^7 has 54 significant bits, the last one is the half-way bit
    v[-4:, :] = 0
    sh[-4:, :] = 0
    v[-4, 0], sh[-4, 0], v[-4, 1], sh[-4, 1] = 1, 60, 1, 7                                     # tie, even below: rounds down
    v[-3, 0], sh[-3, 0], v[-3, 1], sh[-3, 1] = 1, 60, 3, 7                                     # tie, odd below: rounds up
    v[-2, 0], sh[-2, 0], v[-2, 1], sh[-2, 1], v[-2, 2] = 1, 60, 1, 7, 1                        # just above the tie
    v[-1, 0], sh[-1, 0], v[-1, 1], sh[-1, 1], v[-1, 2] = -1, 140, -1, 97, -1                   # negative, across all three words
    unit = rng.integers(-400, 200, n_seq).astype(np.int32)
    unit[-4:] = 0
    words = np.empty((n_seq, 3), dtype=np.uint64)
    out = np.empty(n_seq, dtype=np.uint64)
    v, sh = np.ascontiguousarray(v), np.ascontiguousarray(sh)
    host_emu.host_fixed192(v.ctypes.data_as(ctypes.c_void_p), sh.ctypes.data_as(ctypes.c_void_p), unit.ctypes.data_as(ctypes.c_void_p),
                           words.ctypes.data_as(ctypes.c_void_p), out.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(n_seq),
                           ctypes.c_size_t(length))
    vl, sl, wl = v.tolist(), sh.tolist(), words.tolist()
    want = np.empty(n_seq, dtype=np.float64)
    for i in range(n_seq):
        total = 0
        for x, h in zip(vl[i], sl[i]):
            total += (x << h) if h >= 0 else (x >> -h)
        got = wl[i][0] | (wl[i][1] << 64) | (wl[i][2] << 128)
        assert got == total % (1 << 192), i
        want[i] = float(total)                                       # correctly rounded, ties to even
    want = np.ldexp(want, unit)
    assert np.all(np.isfinite(want)) and not np.any((want != 0) & (np.abs(want) < 2.0 ** -1022))
    assert np.array_equal(out, want.view(np.uint64))
    assert want[-4] == 2.0 ** 60 and want[-3] == 2.0 ** 60 + 2.0 ** 9 and want[-2] == 2.0 ** 60 + 2.0 ** 8


def test_contexts_are_created_selected_and_destroyed_on_the_host():
    """Context plumbing that needs no GPU: a new context has no workspace, selecting it and the default context,
    destroying it (also while it is current)."""
    h1, h2 = lib.ozaki_context_create(), lib.ozaki_context_create()
    assert h1 and h2 and h1 != h2
    lib.ozaki_context_use(h1)
    assert lib.ozaki_last_hip_error() == 0
    f = lib.load().ozaki_dgemm
    assert f(1, 1, 1, 1 << 20, 1, 1 << 20, 1, 1 << 20, 1, 0, 4, 0, 0) == lib.STATUS_WORKSPACE
    lib.ozaki_context_use(h2)
    lib.ozaki_context_destroy(h2)                      # current: the thread falls back to the default context
    assert f(1, 1, 1, 1 << 20, 1, 1 << 20, 1, 1 << 20, 1, 0, 4, 0, 0) == lib.STATUS_WORKSPACE
    lib.ozaki_context_use(None)
    lib.ozaki_context_destroy(h1)
    assert lib.load().ozaki_context_destroy(None) == -1
    assert lib.load().ozaki_context_create(None) == -1


@pytest.fixture(scope="module")
def host_slicer(tmp_path_factory):
    out = tmp_path_factory.mktemp("slicer") / "libhostslicer.so"
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", str(out),
                           os.path.join(ROOT, "tests", "host_slice_element_harness.cpp")])
    return ctypes.CDLL(str(out))


def _host_slice(lib, x, b, s, chunk):
    x = np.ascontiguousarray(x, dtype=np.float64)
    q = np.empty((s, x.size), dtype=np.int32)
    c = np.empty(s, dtype=np.int32)
    rc = lib.host_slice_vector_narrow(x.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(x.size), b, s, chunk,
                                      q.ctypes.data_as(ctypes.c_void_p), c.ctypes.data_as(ctypes.c_void_p))
    return q, c, rc >> 1


@pytest.mark.parametrize("b", [2, 3, 4, 6, 7])
def test_product_narrow_slicer_on_host_equals_oracle(host_slicer, b):
    """The slicer's 32-bit element step (rounding, remainder, the keys that give the next exponent, waiting elements)
    against Eq. 4-8 of the oracle: corner-case vectors, wide-range vectors, short integers (every remainder below
    2^32 units: the keys cannot tell and the lower words decide), several thread sizes."""
    from oracle import ozaki_oracle as oo
    from paper_2508_00441_amd import inputs
    rng = np.random.default_rng(100 + b)
    rho = 53 - b
    k = 200
    X = inputs.nasty_rows(rng, 40, k)
    extra = [
        inputs.phi_matrix(6, k, 6.0, rng),                                         # very wide range: long waits
        rng.integers(-1000, 1001, (4, k)).astype(np.float64),                      # short integers: exhausted early
        np.ldexp(rng.integers(-(1 << 20), 1 << 20, (4, k)).astype(np.float64), -30) + 3.0,      # tiny remainders after slice 1
        np.ldexp(1.0, rng.integers(-40, 40, (4, k))) * np.where(rng.random((4, k)) < 0.5, -1, 1),     # powers of two only
        inputs.phi_matrix(4, k, 1.0, rng) * 2.0 ** -1040,                          # subnormal inputs
    ]
    X = np.vstack([X] + extra)
    X[41, 7] = 0.0
    s = 16
    sl, cs, _ = oo.slice_rows(X, rho, s)
    want_q = np.stack([oo.slice_integers(v, b) for v in sl]).astype(np.int64)      # [s][rows][k]
    want_c = np.stack(cs)                                                          # [s][rows]
    low_decisions = 0
    for r in range(X.shape[0]):
        for chunk in (1, 16, k):
            q, c, low = _host_slice(host_slicer, X[r], b, s, chunk)
            assert np.array_equal(c, want_c[:, r]), (r, chunk, c, want_c[:, r])
            assert np.array_equal(q, want_q[:, r, :]), (r, chunk)
            low_decisions += low
    assert low_decisions > 0                                                       # the fallback of the keys was exercised
