"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: slices, exponents and slice-pair products bit-exact; C bit-exact against the oracle as well,
because the library accumulates in the oracle's order (that is stronger than the required error bound,
which is checked too, against the exact big-integer product).
"""
import math

from fractions import Fraction

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import exact, ozaki_oracle as oz, softfloat  # noqa: E402
from paper_2508_00441_amd import binding as lib, device, inputs  # noqa: E402

FMT = lib.SLICE_FORMATS
ACC = lib.ACCUM_MODES


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lib.load()
    yield
    lib.ozaki_set_workspace(None, 0)


def _gpu_split(X_rows_np, is_B, fmt, s, k_block):
    """X_rows_np: (rows, k) array of the vectors.  Returns codes [T][s] arrays and exps [T][s]."""
    rows, k = X_rows_np.shape
    if is_B:
        Xd = torch.from_numpy(np.ascontiguousarray(X_rows_np)).cuda()            # column-major k x rows, ldx = k
        ldx = k
        ws = device.Workspace.for_problem(0, rows, k, FMT[fmt], s, k_block)
    else:
        Xd = torch.from_numpy(np.ascontiguousarray(X_rows_np.T)).cuda()          # column-major rows x k, ldx = rows
        ldx = rows
        ws = device.Workspace.for_problem(rows, 0, k, FMT[fmt], s, k_block)
    plan = oz.make_plan(k, fmt, k_block)
    T = plan.num_blocks
    dt = torch.int16 if fmt == "fp16" else torch.uint8
    slices = torch.zeros(s * rows * k, dtype=dt, device="cuda")
    exps = torch.zeros(T * s * rows, dtype=torch.int32, device="cuda")
    lib.ozaki_split(int(is_B), rows, k, Xd, ldx, FMT[fmt], s, k_block, slices, exps)
    assert lib.ozaki_last_device_status() == 0
    sl = slices.cpu().numpy()
    if fmt == "fp16":
        sl = sl.view(np.uint16)
    ex = exps.cpu().numpy().reshape(T, s, rows)
    codes = []
    off = 0
    for t in range(T):
        kb_t = min(plan.k_block, k - t * plan.k_block)
        blk = sl[off: off + s * rows * kb_t].reshape(s, rows, kb_t)
        off += s * rows * kb_t
        codes.append(blk)
    ws.close()
    return codes, ex


SPLIT_CASES = [
    # fmt, rows, k, k_block, s, phi
    ("fp8", 256, 256, 0, 12, 0.5),
    ("fp8", 300, 1000, 0, 9, 4.0),        # ragged rows and k (not multiples of the tile / chunk)
    ("fp8", 77, 1000, 384, 7, 2.0),       # three blocks, last one short
    ("fp16", 130, 1024, 0, 8, 1.0),
    ("fp16", 65, 2100, 1024, 6, 2.0),
    ("fp8", 40, 8192, 0, 16, 4.0),        # one workgroup per vector
    ("fp8", 9, 20000, 0, 5, 1.0),         # 1024-thread configuration
    ("fp16", 33, 16384, 4096, 9, 1.0),
    ("fp8", 17, 3, 0, 4, 1.0),            # tiny k
    ("fp16", 40, 200, 0, 6, 1.0),         # b = 8
    ("fp16", 40, 64, 0, 5, 2.0),          # b = 9
    ("fp16", 33, 16, 0, 5, 1.0),          # b = 10
    ("fp16", 19, 700, 256, 5, 2.0),       # b = 8, three blocks
    ("fp6", 256, 256, 0, 12, 0.5),
    ("fp6", 300, 1000, 0, 9, 4.0),        # ragged rows and k
    ("fp6", 77, 1000, 384, 7, 2.0),       # three blocks, last one short
    ("fp6", 40, 8192, 0, 16, 4.0),
    ("fp6", 9, 20000, 0, 5, 1.0),
    ("fp6", 17, 3, 0, 4, 1.0),
    ("fp6_e3m2", 300, 1000, 0, 9, 4.0),
    ("fp6_e3m2", 77, 1000, 384, 7, 2.0),
    ("fp6_e3m2", 9, 20000, 0, 5, 1.0),
]


@pytest.mark.parametrize("fmt,rows,k,k_block,s,phi", SPLIT_CASES)
@pytest.mark.parametrize("is_B", [0, 1])
def test_split_is_bit_exact(fmt, rows, k, k_block, s, phi, is_B):
    rng = np.random.default_rng(100 + rows + k)
    X = inputs.phi_matrix(rows, k, phi, rng)
    X[0, :] = 0.0
    if rows > 3:
        X[1, :] = 1.0
        X[2, :] = np.nextafter(1.0, 2.0)
        X[3, : k // 2] = 0.0
    if rows > 5:
        X[4, :] *= 2.0 ** -1040            # subnormal inputs are still sliced exactly
        X[5, :] *= 2.0 ** 600
    ref_codes, ref_exps, plan = oz.split_operand(X, fmt, s, k_block)
    got_codes, got_exps = _gpu_split(X, is_B, fmt, s, k_block)
    for t in range(plan.num_blocks):
        for p in range(s):
            assert np.array_equal(got_exps[t][p], ref_exps[t][p]), (t, p)
            assert np.array_equal(got_codes[t][p], ref_codes[t][p]), (t, p)


def _upload(A, B):
    return device.to_device_colmajor(A), device.to_device_colmajor(B)


PRODUCT_CASES = [
    ("fp8", 256, 256, 256, 0, 12, 0.5),
    ("fp8", 300, 270, 520, 0, 6, 2.0),
    ("fp8", 100, 600, 1000, 384, 5, 4.0),
    ("fp16", 260, 130, 1100, 512, 5, 1.0),
    ("fp16", 64, 64, 4096, 0, 4, 1.0),
    ("fp6", 256, 256, 256, 0, 12, 0.5),
    ("fp6", 300, 270, 520, 0, 6, 2.0),
    ("fp6", 100, 600, 1000, 384, 5, 4.0),
    ("fp6", 515, 260, 4096, 0, 3, 1.0),
    ("fp6_e3m2", 300, 270, 520, 0, 6, 2.0),
    ("fp6_e3m2", 100, 600, 1000, 384, 5, 4.0),
    ("fp6_e3m2", 130, 70, 32768, 0, 3, 0.5),         # long inner dimension: sums up to 2^21 units
]


@pytest.mark.parametrize("fmt,m,n,k,k_block,s,phi", PRODUCT_CASES)
def test_pair_products_are_bit_exact(fmt, m, n, k, k_block, s, phi):
    A, B = inputs.phi_pair(m, n, k, phi, seed=m + n + k)
    Ad, Bd = _upload(A, B)
    plan = oz.make_plan(k, fmt, k_block)
    T, npairs = plan.num_blocks, s * (s + 1) // 2
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block)
    P = torch.full((T, npairs, n, m), float("nan"), dtype=torch.float32, device="cuda")
    lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT[fmt], s, k_block, P)
    assert lib.ozaki_last_device_status() == 0
    Pn = P.cpu().numpy()
    _, blocks = oz.ozaki_dgemm(A, B, fmt, s, k_block, return_blocks=True, accumulate="runs")
    for t, br in enumerate(blocks):
        assert br.pairs == oz.pair_order(s)
        for z, Pref in enumerate(br.products):
            want = np.ldexp(Pref.astype(np.float64), -2 * plan.b).astype(np.float32).T     # (n, m)
            assert np.array_equal(Pn[t, z], want), (t, z)
    ws.close()


DGEMM_CASES = [
    # fmt, m, n, k, k_block, s, phi
    ("fp8", 256, 256, 256, 0, 12, 0.5),          # the small benchmark configuration
    ("fp8", 300, 270, 520, 0, 15, 4.0),          # ragged, wide exponent range
    ("fp8", 100, 600, 1000, 384, 12, 2.0),       # k-blocked, short last block
    ("fp16", 260, 130, 1100, 512, 7, 1.0),
    ("fp16", 512, 256, 2048, 1024, 8, 1.0),
    ("fp8", 513, 255, 2048, 0, 13, 1.0),
    ("fp8", 16, 16, 16, 0, 3, 1.0),
    ("fp6", 256, 256, 256, 0, 12, 0.5),
    ("fp6", 300, 270, 520, 0, 15, 4.0),
    ("fp6", 100, 600, 1000, 384, 12, 2.0),
    ("fp6", 513, 255, 2048, 0, 13, 1.0),
    ("fp6_e3m2", 300, 270, 520, 0, 17, 2.0),
    ("fp6_e3m2", 100, 600, 1000, 384, 15, 1.0),
    # few tiles, long k (64 or more stages per pair): the plan shortens the GEMM kernel's groups
    ("fp8", 300, 270, 5000, 0, 11, 1.0),
    ("fp6", 260, 500, 9000, 4608, 11, 1.0),
    ("fp16", 300, 130, 4100, 2050, 8, 1.0),
]


@pytest.mark.parametrize("fmt,m,n,k,k_block,s,phi", DGEMM_CASES)
@pytest.mark.parametrize("accum", ["hw", "emu"])
def test_dgemm_matches_oracle(fmt, m, n, k, k_block, s, phi, accum):
    A, B = inputs.phi_pair(m, n, k, phi, seed=7 * m + n + k)
    Ad, Bd = _upload(A, B)
    ldc = m + 3
    Cd = torch.full((n, ldc), float("nan"), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block)
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, ldc, FMT[fmt], s, k_block, ACC[accum])
    assert lib.ozaki_last_device_status() == 0
    Cfull = Cd.cpu().numpy()
    C = Cfull[:, :m].T
    assert np.all(np.isnan(Cfull[:, m:]))                         # the padding of ldc is not touched
    Cref = oz.ozaki_dgemm(A, B, fmt, s, k_block, accumulate="runs")
    assert np.array_equal(C.view(np.uint64), Cref.view(np.uint64))
    # the stated bound against the exact product, on sampled entries, next to a native FP64 GEMM
    ent = exact.sample_entries(m, n, 12, seed=m)
    e_ab, e_c, _, _ = exact.sampled_errors(A, B, ent, [C[i, j] for i, j in ent])
    if s >= 7:
        assert e_ab <= 4 * k * 2.0 ** -53
    ws.close()


@pytest.mark.parametrize("fmt,k_block", [("fp8", 0), ("fp6", 0), ("fp16", 256)])
def test_operands_off_the_16_byte_boundary_with_odd_leading_dimensions(fmt, k_block):
    """A, B and C start one element (8 bytes) past a 16-byte boundary and have odd leading dimensions: the split
    kernel's two-element loads are not allowed there, the result must not change."""
    m, n, k, s = 270, 140, 600, 9
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=99)
    lda, ldb, ldc = m + 1, k + 1, m + 1
    bufA = torch.zeros(1 + k * lda, dtype=torch.float64, device="cuda")
    bufB = torch.zeros(1 + n * ldb, dtype=torch.float64, device="cuda")
    bufC = torch.full((1 + n * ldc,), float("nan"), dtype=torch.float64, device="cuda")
    bufA[1:].view(k, lda)[:, :m] = torch.from_numpy(np.ascontiguousarray(A.T)).cuda()     # column-major m x k
    bufB[1:].view(n, ldb)[:, :k] = torch.from_numpy(np.ascontiguousarray(B.T)).cuda()     # column-major k x n
    Ad, Bd, Cd = bufA[1:], bufB[1:], bufC[1:]
    assert Ad.data_ptr() % 16 == 8 and Bd.data_ptr() % 16 == 8
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block)
    for accum in ("hw", "emu"):
        Cd.fill_(float("nan"))
        lib.ozaki_dgemm(m, n, k, Ad, lda, Bd, ldb, Cd, ldc, FMT[fmt], s, k_block, ACC[accum])
        assert lib.ozaki_last_device_status() == 0
        Cfull = Cd.view(n, ldc).cpu().numpy()
        assert np.all(np.isnan(Cfull[:, m:])) and np.isnan(float(bufC[0]))
        Cref = oz.ozaki_dgemm(A, B, fmt, s, k_block, accumulate="runs")
        assert np.array_equal(np.ascontiguousarray(Cfull[:, :m].T).view(np.uint64), Cref.view(np.uint64))
    ws.close()


def test_slice_count_until_exhaustion_and_error_free_product():
    """The paper's own stopping rule (slice until the remainder is zero) and its consequence: with that many
    slices and all pairs, the pair products sum to the exact product (Eq. 9-10)."""
    rng = np.random.default_rng(77)
    cases = [
        ("fp8", inputs.uniform_1_10(70, 300, rng), 0),
        ("fp8", inputs.phi_matrix(33, 1000, 1.0, rng), 384),
        ("fp16", inputs.uniform_1_10(40, 2100, rng), 1024),
        ("fp6", inputs.full_mantissa_one_binade(20, 512, rng), 0),
        ("fp8", np.round(rng.uniform(-16, 16, (10, 64))) * 2.0 ** 7, 0),       # integers: one slice
        ("fp8", np.zeros((5, 40)), 0),
        ("fp16", inputs.phi_matrix(9, 64, 6.0, rng), 0),
        ("fp8", inputs.phi_matrix(9, 64, 30.0, np.random.default_rng(5)), 0),   # exponent range too wide for 32 slices
    ]
    for fmt, X, kb in cases:
        rows, k = X.shape
        want = oz.count_slices_to_exhaustion(X, fmt, kb)
        for is_B in (0, 1):
            Xd = torch.from_numpy(np.ascontiguousarray(X if is_B else X.T)).cuda()      # column-major k x rows / rows x k
            ws = device.Workspace(256 + 8 * rows * k + 256)
            got = lib.ozaki_count_slices(is_B, rows, k, Xd, k if is_B else rows, FMT[fmt], kb)
            ws.close()
            assert got == min(want, lib.MAX_SLICES + 1), (fmt, rows, k, kb, is_B, got, want)
    # error-free product on a small case: every entry of C is the correctly rounded exact value
    A = inputs.uniform_1_10(40, 96, rng)
    B = inputs.uniform_1_10(96, 24, rng)
    Ad, Bd = _upload(A, B)
    ws = device.Workspace(1 << 20)
    s = max(lib.ozaki_count_slices(0, 40, 96, Ad, 40, FMT["fp8"], 0), lib.ozaki_count_slices(1, 24, 96, Bd, 96, FMT["fp8"], 0))
    ws.close()
    assert s == max(oz.count_slices_to_exhaustion(A, "fp8"), oz.count_slices_to_exhaustion(B.T.copy(), "fp8")) <= lib.MAX_SLICES
    ws = device.Workspace.for_problem(40, 24, 96, FMT["fp8"], s | lib.PAIRS_ALL, 0)
    Cd = torch.empty((24, 40), dtype=torch.float64, device="cuda")
    lib.ozaki_dgemm(40, 24, 96, Ad, 40, Bd, 96, Cd, 40, FMT["fp8"], s | lib.PAIRS_ALL, 0, ACC["emu"])
    C = Cd.cpu().numpy().T
    ws.close()
    assert np.array_equal(C.view(np.uint64), oz.ozaki_dgemm(A, B, "fp8", s, 0, mode="full", accumulate="runs").view(np.uint64))
    for i in range(0, 40, 7):
        for j in range(0, 24, 5):
            ex = exact.exact_dot(A[i, :], B[:, j])
            assert abs(Fraction(float(C[i, j])) - ex) <= Fraction(float(np.spacing(abs(C[i, j])))) , (i, j)


@pytest.mark.parametrize("accum", ["hw", "emu"])
@pytest.mark.parametrize("fmt,m,n,k,k_block,s", [("fp8", 300, 270, 520, 0, 9), ("fp16", 130, 260, 700, 256, 5), ("fp6", 257, 64, 1000, 384, 8)])
def test_scaled_dgemm_matches_oracle(fmt, m, n, k, k_block, s, accum):
    """C = alpha (A B) + beta C: one rounded multiplication per term, one rounded addition, bit for bit."""
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=m + 3 * n + k)
    rng = np.random.default_rng(m * n)
    C0 = inputs.phi_matrix(m, n, 2.0, rng)
    Ad, Bd = _upload(A, B)
    ldc = m + 5
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block, scaled=True)
    P = oz.ozaki_dgemm(A, B, fmt, s, k_block, accumulate="runs")
    for alpha, beta in ((-2.5, 0.0), (1.0, 1.0), (0.3, -1.7), (0.0, 2.0), (1.0, 0.0)):
        Cfull = np.full((n, ldc), np.nan)
        if beta != 0.0:
            Cfull[:, :m] = C0.T
        Cd = torch.from_numpy(Cfull).cuda()
        lib.ozaki_dgemm_scaled(m, n, k, alpha, Ad, m, Bd, k, beta, Cd, ldc, FMT[fmt], s, k_block, ACC[accum])
        assert lib.ozaki_last_device_status() == 0
        out = Cd.cpu().numpy()
        assert np.all(np.isnan(out[:, m:]))
        want = oz.ozaki_dgemm(A, B, fmt, s, k_block, alpha=alpha, beta=beta, C0=C0, accumulate="runs")
        assert np.array_equal(out[:, :m].T.view(np.uint64), want.view(np.uint64)), (alpha, beta)
        if (alpha, beta) == (1.0, 0.0):
            assert np.array_equal(want.view(np.uint64), P.view(np.uint64))
    # k = 0: the product is the zero matrix
    Cd = torch.from_numpy(np.ascontiguousarray(C0.T)).cuda()
    lib.ozaki_dgemm_scaled(m, n, 0, 3.0, Ad, m, Bd, 1, 0.5, Cd, m, FMT[fmt], s, k_block, ACC[accum])
    assert np.array_equal(Cd.cpu().numpy().T.view(np.uint64), (3.0 * np.zeros((m, n)) + 0.5 * C0).view(np.uint64))
    ws.close()


@pytest.mark.parametrize("fmt,m,n,k,k_block,s,phi", [("fp8", 300, 270, 520, 0, 7, 1.0), ("fp16", 130, 260, 700, 256, 5, 2.0),
                                                     ("fp8", 64, 64, 4096, 0, 11, 0.5),
                                                     ("fp8", 70, 50, 200, 0, 32, 6.0),        # the largest slice count
                                                     ("fp6", 70, 50, 200, 64, 32, 6.0)])
@pytest.mark.parametrize("accum", ["hw", "emu"])
def test_all_pairs_mode_matches_oracle(fmt, m, n, k, k_block, s, phi, accum):
    """num_slices | PAIRS_ALL: all s*s slice pairs (the paper's setting), anti-diagonals 2s ... 2."""
    A, B = inputs.phi_pair(m, n, k, phi, seed=m + 3 * n)
    Ad, Bd = _upload(A, B)
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s | lib.PAIRS_ALL, k_block)
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s | lib.PAIRS_ALL, k_block, ACC[accum])
    assert lib.ozaki_last_device_status() == 0
    C = device.from_device_colmajor(Cd)
    Cref, blocks = oz.ozaki_dgemm(A, B, fmt, s, k_block, mode="full", return_blocks=True, accumulate="runs")
    assert np.array_equal(C.view(np.uint64), Cref.view(np.uint64))
    if accum == "hw":
        T, npairs = len(blocks), s * s
        P = torch.zeros((T, npairs, n, m), dtype=torch.float32, device="cuda")
        lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT[fmt], s | lib.PAIRS_ALL, k_block, P)
        torch.cuda.synchronize()
        Pn = P.cpu().numpy()
        b = oz.make_plan(k, fmt, k_block).b
        for t, br in enumerate(blocks):
            assert br.pairs == oz.pair_order(s, "full")
            for z, Pref in enumerate(br.products):
                assert np.array_equal(Pn[t, z], np.ldexp(Pref.astype(np.float64), -2 * b).astype(np.float32).T), (t, z)
    ws.close()


def test_chunked_workspace_gives_identical_bits():
    fmt, m, n, k, s = "fp8", 300, 270, 520, 8
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=5)
    Ad, Bd = _upload(A, B)
    outs = []
    for minimum in (False, True):
        ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, 0, minimum=minimum)
        for accum in ("hw", "emu"):
            Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
            lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, 0, ACC[accum])
            torch.cuda.synchronize()
            outs.append(Cd.cpu().numpy().view(np.uint64))
        ws.close()
    assert all(np.array_equal(outs[0], o) for o in outs[1:])
    # and repeated runs are reproducible bit for bit
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, 0)
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, 0, ACC["hw"])
    assert np.array_equal(Cd.cpu().numpy().view(np.uint64), outs[0])
    ws.close()


def test_emulated_add_is_bitwise_hardware_on_device():
    rng = np.random.default_rng(77)
    n = 4_000_000

    def rnd(n, lo, hi):
        frac = rng.integers(0, 1 << 52, n, dtype=np.uint64)
        e = rng.integers(lo + 1023, hi + 1023, n, dtype=np.uint64)
        sg = rng.integers(0, 2, n, dtype=np.uint64)
        return ((sg << np.uint64(63)) | (e << np.uint64(52)) | frac).view(np.float64)

    a = rnd(3 * n, -300, 300)
    b = np.concatenate([
        rnd(n, -300, 300),
        np.ldexp(rnd(n, -1, 1), np.frexp(a[n:2 * n])[1] + rng.integers(-70, 71, n)),
        -a[2 * n:] * (1.0 + np.ldexp(rng.integers(-8, 9, n).astype(np.float64), -rng.integers(30, 53, n))),
    ])
    a[:4] = [0.0, 1.5, 0.0, -2.5]
    b[:4] = [0.0, 0.0, -3.0, 2.5]
    ad, bd = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
    out = torch.empty_like(ad)
    lib.ozaki_set_stream(torch.cuda.current_stream().cuda_stream)
    lib.ozaki_fp64_add_emulated(ad, bd, out, a.size)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got.view(np.uint64), (a + b).view(np.uint64))
    assert np.array_equal(got.view(np.uint64), (ad + bd).cpu().numpy().view(np.uint64))     # the GPU's own FP64 adder


def test_edge_cases_and_error_paths():
    m, n, k = 48, 32, 64
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=1)
    Ad, Bd = _upload(A, B)
    Cd = torch.full((n, m), 7.0, dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, 0, 4, 0)
    # empty problems succeed and leave C alone; k = 0 zeroes C
    assert lib.ozaki_dgemm(0, n, k, Ad, 1, Bd, k, Cd, 1, 0, 4, 0, 0) == 0
    assert lib.ozaki_dgemm(m, 0, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0) == 0
    torch.cuda.synchronize()
    assert float(Cd.min()) == 7.0
    assert lib.ozaki_dgemm(m, n, 0, Ad, m, Bd, 1, Cd, m, 0, 4, 0, 0) == 0
    torch.cuda.synchronize()
    assert float(Cd.abs().max()) == 0.0
    # argument errors: nothing is launched
    assert lib.ozaki_dgemm(-1, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0, check=False) == -1
    assert lib.ozaki_dgemm(m, n, k, Ad, m - 1, Bd, k, Cd, m, 0, 4, 0, 0, check=False) == -5
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k - 1, Cd, m, 0, 4, 0, 0, check=False) == -7
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m - 1, 0, 4, 0, 0, check=False) == -9
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 9, 4, 0, 0, check=False) == -10
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 2, check=False) == -13
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 33, 0, 0, check=False) == lib.STATUS_INFEASIBLE
    # workspace too small
    ws.close()
    small = device.Workspace(4096)
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0, check=False) == lib.STATUS_WORKSPACE
    small.close()
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0, check=False) == lib.STATUS_WORKSPACE
    # non-finite input raises the device flag once
    ws = device.Workspace.for_problem(m, n, k, 0, 4, 0)
    A2 = A.copy()
    A2[3, 5] = np.inf
    A2d = device.to_device_colmajor(A2)
    lib.ozaki_dgemm(m, n, k, A2d, m, Bd, k, Cd, m, 0, 4, 0, 0)
    assert lib.ozaki_last_device_status() == lib.STATUS_NONFINITE
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0)
    assert lib.ozaki_last_device_status() == 0
    # default number of slices (data-independent heuristic; parity unpinned): still inside the bound
    ws.close()
    ws = device.Workspace.for_problem(m, n, k, 0, 0, 0)
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 0, 0, 0)
    torch.cuda.synchronize()
    C = device.from_device_colmajor(Cd)
    ent = exact.sample_entries(m, n, 10, seed=2)
    assert exact.sampled_errors(A, B, ent, [C[i, j] for i, j in ent])[0] <= 4 * k * 2.0 ** -53
    ws.close()


def test_one_slice_integer_inputs_reproduce_integer_gemm():
    rng = np.random.default_rng(3)
    m, n, k = 70, 90, 200
    QA = rng.integers(-16, 17, (m, k))
    QB = rng.integers(-16, 17, (k, n))
    QA[:, 0] = 16
    QB[0, :] = -16
    A = np.ldexp(QA.astype(np.float64), rng.integers(-20, 20, m)[:, None])
    B = np.ldexp(QB.astype(np.float64), rng.integers(-20, 20, n)[None, :])
    Ad, Bd = _upload(A, B)
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, 0, 1, 0)
    for accum in (0, 1):
        lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 1, 0, accum)
        torch.cuda.synchronize()
        assert np.array_equal(device.from_device_colmajor(Cd), A @ B)       # A @ B is exact here
    ws.close()


def test_products_at_the_edge_of_the_fp32_window():
    """k_block * 4^b = 2^24 with every entry at the row maximum: each product is exactly +-2^24 units."""
    m, n, k = 40, 24, 2048
    A = np.ones((m, k))
    B = np.ones((k, n))
    B[:, ::2] = -1.0
    Ad, Bd = _upload(A, B)
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT["fp16"], 2, 1024)
    for accum in (0, 1):
        lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT["fp16"], 2, 1024, accum)
        torch.cuda.synchronize()
        assert np.array_equal(device.from_device_colmajor(Cd), A @ B)
    P = torch.zeros((2, 3, n, m), dtype=torch.float32, device="cuda")
    lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT["fp16"], 2, 1024, P)
    torch.cuda.synchronize()
    Pn = P.cpu().numpy()
    assert np.array_equal(np.abs(Pn[:, 2]), np.full((2, n, m), 1024.0, dtype=np.float32))   # pair (1,1): 2^24 * 2^-14
    ws.close()


@pytest.mark.parametrize("fmt,b", [("fp8", 4), ("fp6", 4), ("fp6_e3m2", 3)])
def test_narrow_formats_at_the_edge_of_the_fp32_window(fmt, b):
    """Every entry at the row maximum and the longest block the library takes: each product is +-k * 4^b units."""
    m, n, k = 40, 24, 32768
    A = np.ones((m, k))
    B = np.ones((k, n))
    B[:, ::2] = -1.0
    Ad, Bd = _upload(A, B)
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], 2, 0)
    assert lib.ozaki_plan(k, FMT[fmt])[1] == b
    for accum in (0, 1):
        lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], 2, 0, accum)
        torch.cuda.synchronize()
        assert np.array_equal(device.from_device_colmajor(Cd), A @ B)
    P = torch.zeros((1, 3, n, m), dtype=torch.float32, device="cuda")
    lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT[fmt], 2, 0, P)
    torch.cuda.synchronize()
    assert np.array_equal(np.abs(P.cpu().numpy()[0, 2]), np.full((n, m), float(k), dtype=np.float32))      # pair (1,1)
    ws.close()


_INPUT_CACHE = {}


def _config_inputs(cfg):
    """Inputs of a benchmark configuration (seed 0), uploaded once per shape/phi and reused by the variants."""
    key = (cfg["m"], cfg["n"], cfg["k"], cfg["phi"])
    if key not in _INPUT_CACHE:
        _INPUT_CACHE.clear()
        torch.cuda.empty_cache()
        A, B = inputs.phi_pair(cfg["m"], cfg["n"], cfg["k"], cfg["phi"], seed=0)
        _INPUT_CACHE[key] = (A, B) + _upload(A, B)
    return _INPUT_CACHE[key]


@pytest.mark.parametrize("name", ["c2_4096_fp8_hw", "c3_8192_fp8_emu", "c5a_16384x1024_fp8", "c5b_1024x65536_fp8",
                                  "c4_16384_fp16_kb1024", "c4_16384_fp16_kb4096", "c4_16384_fp8"])
def test_full_size_configs_on_sampled_rows_and_columns(name):
    """At the benchmark's sizes the oracle cannot form all of C; rows of A and columns of B are sliced
    independently of each other, so the oracle run on a few rows and columns must reproduce exactly the
    corresponding entries of the device result (in the launch configuration bench.py times)."""
    cfg = inputs.CONFIGS[name]
    m, n, k, fmt, kb = cfg["m"], cfg["n"], cfg["k"], cfg["fmt"], cfg["k_block"]
    s = inputs.NUM_SLICES[name]
    print(f"config {name}: m={m} n={n} k={k} fmt={fmt} k_block={kb} s={s}", flush=True)
    A, B, Ad, Bd = _config_inputs(cfg)
    Cd = torch.empty((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, kb)
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, kb, ACC[cfg["accum"]])
    assert lib.ozaki_last_device_status() == 0
    rng = np.random.default_rng(42)
    ns = 24 if k <= 16384 else 12
    rows = np.sort(rng.choice(m, ns, replace=False))
    cols = np.sort(rng.choice(n, ns, replace=False))
    rows[0], cols[-1] = 0, n - 1
    Csub = Cd[torch.from_numpy(cols).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy().T
    Cref = oz.ozaki_dgemm(A[rows, :], B[:, cols], fmt, s, kb, accumulate="runs")
    assert np.array_equal(Csub.view(np.uint64), Cref.view(np.uint64))
    ent = [(int(i), int(j)) for i, j in zip(rng.integers(0, ns, 8), rng.integers(0, ns, 8))]
    got = [Csub[i, j] for i, j in ent]
    e_ab, e_c, _, _ = exact.sampled_errors(A[rows, :], B[:, cols], ent, got)
    assert e_ab <= 4 * k * 2.0 ** -53
    ws.close()
    del Cd, ws
    torch.cuda.empty_cache()


def test_dgemm_can_be_captured_in_a_hip_graph_and_replayed():
    """ozaki_dgemm only enqueues kernels on the library stream (no allocation, no synchronisation, no memset), so a
    caller can capture it; every replay must give the eager result, also with other work between the replays."""
    m, n, k, s = 300, 270, 520, 9
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=11)
    A2, B2 = inputs.phi_pair(m, n, k, 2.0, seed=12)
    Ad, Bd = _upload(A, B)
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT["fp8"], s, 0)
    want = [oz.ozaki_dgemm(A, B, "fp8", s, 0, accumulate="runs"), oz.ozaki_dgemm(A2, B2, "fp8", s, 0, accumulate="runs")]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        lib.ozaki_set_stream(side.cuda_stream)
        lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT["fp8"], s, 0, ACC["emu"])      # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT["fp8"], s, 0, ACC["emu"])
    torch.cuda.synchronize()
    for rep in range(4):
        src = (A, B) if rep % 2 == 0 else (A2, B2)
        Ad.copy_(torch.from_numpy(np.ascontiguousarray(src[0].T)).cuda())                 # eager work between the replays
        Bd.copy_(torch.from_numpy(np.ascontiguousarray(src[1].T)).cuda())
        Cd.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Cd.cpu().numpy().T
        assert np.array_equal(got.view(np.uint64), want[rep % 2].view(np.uint64)), rep
    lib.ozaki_set_stream(torch.cuda.current_stream().cuda_stream)
    assert lib.ozaki_last_device_status() == 0
    ws.close()


def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        fmt = ["fp8", "fp16", "fp6", "fp6_e3m2"][int(rng.integers(0, 4))]
        m, n = int(rng.integers(1, 400)), int(rng.integers(1, 400))
        k = int(rng.integers(1, 3000))
        kb = [0, int(rng.integers(1, k + 1)), int(rng.integers(1, 200))][int(rng.integers(0, 3))]
        s = int(rng.integers(1, 11))
        full = bool(rng.integers(0, 2)) and s <= 7
        phi = float(rng.choice([0.5, 1.0, 3.0]))
        accum = ["hw", "emu"][int(rng.integers(0, 2))]
        cases.append((fmt, m, n, k, kb, s, full, phi, accum))
    return cases


@pytest.mark.parametrize("fmt,m,n,k,kb,s,full,phi,accum", _random_cases(24, seed=2025))
def test_random_shapes_and_parameters_match_oracle(fmt, m, n, k, kb, s, full, phi, accum):
    """Seeded random problem shapes, block lengths (any value, also shorter than a chunk), slice counts, pair sets and
    formats: C bit-identical to the oracle."""
    A, B = inputs.phi_pair(m, n, k, phi, seed=m * 7 + n * 3 + k)
    Ad, Bd = _upload(A, B)
    s_arg = s | lib.PAIRS_ALL if full else s
    Cd = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s_arg, kb)
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s_arg, kb, ACC[accum])
    assert lib.ozaki_last_device_status() == 0
    C = device.from_device_colmajor(Cd)
    ws.close()
    Cref = oz.ozaki_dgemm(A, B, fmt, s, kb, mode="full" if full else "triangle", accumulate="runs")
    assert np.array_equal(C.view(np.uint64), Cref.view(np.uint64))
