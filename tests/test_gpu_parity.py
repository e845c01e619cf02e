"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: slices, exponents and slice-pair products (each pair on its own, and the exact run sums of the chained launch
configuration) bit-exact.  C bit-exact against the oracle for each of the three accumulation rules: the plain
term-by-term FP64 sum of Eq. 10 (OZAKI_SUM_PLAIN), the equal-scale-run variant the library uses by default
(OZAKI_SUM_RUNS) and the fixed-point sum rounded once (OZAKI_ACCUM_EXACT_FIXED).  The default mode is also measured
against the plain oracle (error no larger, distance in units in the last place), and everything against the stated
bound 4 k 2^-53 relative to the exact product.
"""
import math

from fractions import Fraction

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import exact, formats, ozaki_oracle as oz, softfloat  # noqa: E402
from paper_2508_00441_amd import binding as lib, device, inputs  # noqa: E402

FMT = lib.SLICE_FORMATS
ACC = lib.ACCUM_MODES
PAIRS = lib.PAIR_SETS
SUM = lib.SUM_RULES
BOUND = lambda k: 4 * k * 2.0 ** -53           # noqa: E731  (the tolerance the benchmark spec states for C)


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
    slices = torch.full((s * rows * k,), 0x55, dtype=dt, device="cuda")
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
    ("int8", 300, 1000, 0, 9, 4.0),
    ("int8", 77, 1000, 384, 7, 2.0),
    ("int8", 9, 20000, 0, 5, 1.0),
    ("fp8", 5, 16384, 0, 6, 1.0),         # the longest block of the register-resident kernel
    ("fp6", 5, 16384, 0, 6, 1.0),
    ("fp16", 5, 16384, 0, 6, 1.0),
    ("fp6", 9, 30000, 0, 5, 1.0),
    # blocks longer than the register-resident kernel takes (Table 2's last rows: b = 4 at 65536, b = 3 beyond)
    ("fp8", 5, 65536, 0, 6, 2.0),
    ("fp8", 3, 131072, 0, 5, 1.0),
    ("fp6", 3, 70000, 40000, 5, 1.0),
    ("fp16", 3, 65536, 0, 4, 1.0),
    ("int8", 2, 262144, 0, 4, 1.0),
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


def _random_split_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        fmt = ["fp8", "fp6", "fp6_e3m2", "int8", "fp16"][int(rng.integers(0, 5))]
        rows = int(rng.integers(1, 600))
        k = int(rng.choice([int(rng.integers(1, 200)), int(rng.integers(200, 5000)), int(rng.integers(5000, 20000))]))
        kb = [0, int(rng.integers(1, k + 1))][int(rng.integers(0, 2))]
        if fmt == "fp16" and (kb or k) > 16384:
            kb = 4096                                    # the longest FP16 block with an exact FP32 window is 16384 (b = 5)
        cases.append((fmt, rows, k, kb, int(rng.integers(1, 20)), float(rng.choice([0.5, 2.0, 4.0, 8.0])), int(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("fmt,rows,k,k_block,s,phi,is_B", _random_split_cases(36, seed=99))
def test_split_of_random_shapes_is_bit_exact(fmt, rows, k, k_block, s, phi, is_B):
    """Seeded random vector counts, lengths (up to blocks that go to the streaming kernel), block lengths, slice counts
    and value ranges, all formats: codes and exponents bit-identical to the oracle."""
    test_split_is_bit_exact(fmt, rows, k, k_block, s, phi, is_B)


@pytest.mark.parametrize("fmt,k,k_block,s", [("fp8", 64, 0, 9), ("fp8", 4096, 0, 12), ("fp6", 777, 300, 9), ("fp6_e3m2", 64, 0, 12),
                                             ("int8", 1000, 0, 8), ("fp16", 200, 0, 6), ("fp16", 64, 0, 5), ("fp16", 16, 0, 5),
                                             ("fp16", 1024, 0, 7), ("fp8", 40000, 0, 9)])
@pytest.mark.parametrize("is_B", [0, 1])
def test_split_of_the_corner_case_rows_is_bit_exact(fmt, k, k_block, s, is_B):
    """The rows the oracle's own pins use: zero vector, power-of-two maxima, exact ties of the rounding, a 2^300 outlier
    (elements that wait many slices before they reach the slice unit; with FP16 slices of 8 and more bits the branch
    that rounds an element in its integer form), a row scaled by 2^-400, full significands with random signs."""
    rng = np.random.default_rng(11 + k)
    X = inputs.nasty_rows(rng, 12, k)
    X[9, :] = X[6, :]
    X[9, 3] = 2.0 ** 300                                  # full significands next to an outlier
    X[10, :] = np.ldexp(X[8, :], 77)                      # the tie row again, scaled
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
    ("int8", 300, 270, 520, 0, 6, 2.0),
    ("int8", 100, 600, 1000, 384, 5, 4.0),
    ("int8", 130, 70, 32768, 0, 3, 0.5),
]


def _oracle_products(A, B, fmt, s, k_block, mode="triangle"):
    plan = oz.make_plan(A.shape[1], fmt, k_block)
    _, blocks = oz.ozaki_dgemm(A, B, fmt, s, k_block, mode=mode, return_blocks=True)
    return plan, blocks


def _as_device_words(P_int, fmt, b):
    """The oracle's exact integer products as the 4-byte words the device must hold, transposed to (n, m)."""
    if fmt == "int8":
        return P_int.astype(np.int32).T
    return np.ldexp(P_int.astype(np.float64), -2 * b).astype(np.float32).T


@pytest.mark.parametrize("fmt,m,n,k,k_block,s,phi", PRODUCT_CASES)
def test_pair_products_are_bit_exact(fmt, m, n, k, k_block, s, phi):
    A, B = inputs.phi_pair(m, n, k, phi, seed=m + n + k)
    Ad, Bd = _upload(A, B)
    plan, blocks = _oracle_products(A, B, fmt, s, k_block)
    T, npairs = plan.num_blocks, s * (s + 1) // 2
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block)
    dt = torch.int32 if fmt == "int8" else torch.float32
    P = torch.full((T, npairs, n, m), -77, dtype=dt, device="cuda")
    L = torch.full((T, npairs, n, m), 99, dtype=torch.uint8, device="cuda")
    lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT[fmt], s, k_block, P, run_len_out=L)
    assert lib.ozaki_last_device_status() == 0
    Pn = P.cpu().numpy()
    assert int(L.min()) == 1 and int(L.max()) == 1            # nothing is chained in this mode
    for t, br in enumerate(blocks):
        assert br.pairs == oz.pair_order(s)
        for z, Pref in enumerate(br.products):
            assert np.array_equal(Pn[t, z], _as_device_words(Pref, fmt, plan.b)), (t, z)
    ws.close()


CHAIN_CASES = [
    # fmt, m, n, k, k_block, s, mode, input recipe
    ("fp8", 300, 270, 520, 0, 8, "triangle", "phi1"),
    ("fp8", 300, 270, 520, 0, 9, "triangle", "phi4"),          # wide rows: irregular exponent ladders break the runs
    ("fp8", 515, 260, 2048, 0, 6, "full", "binade"),           # one-binade rows: regular ladders, long runs (window: 32 pairs)
    ("fp8", 130, 200, 8192, 0, 12, "triangle", "u110"),        # window of 8 pairs: anti-diagonals are cut into groups
    ("fp16", 260, 130, 700, 256, 5, "triangle", "phi1"),       # FP16, b = 8: the window holds one pair, nothing may chain
    ("fp16", 200, 100, 64, 16, 6, "triangle", "binade"),       # FP16, b = 10 at 16 elements: window of 1 as well
    ("fp6", 300, 270, 520, 0, 8, "triangle", "phi1"),
    ("fp6_e3m2", 257, 300, 1000, 384, 9, "full", "u110"),
    ("int8", 300, 270, 520, 0, 7, "triangle", "phi1"),         # INT32 window: whole anti-diagonals chain
    ("int8", 257, 100, 3000, 0, 8, "full", "binade"),
]


def _recipe(name, m, n, k, seed):
    rng = np.random.default_rng(seed)
    if name == "u110":
        return inputs.uniform_1_10(m, k, rng), inputs.uniform_1_10(k, n, rng)
    if name == "binade":
        sa = np.where(rng.random((m, k)) < 0.5, -1.0, 1.0)
        sb = np.where(rng.random((k, n)) < 0.5, -1.0, 1.0)
        A = inputs.full_mantissa_one_binade(m, k, rng) * sa * np.ldexp(1.0, rng.integers(-9, 9, m))[:, None]
        B = inputs.full_mantissa_one_binade(k, n, rng) * sb * np.ldexp(1.0, rng.integers(-9, 9, n))[None, :]
        A[m // 2, :] = inputs.phi_matrix(1, k, 3.0, rng)[0]      # one irregular row among regular ones
        return A, B
    return inputs.phi_pair(m, n, k, float(name[3:]), seed=seed)


@pytest.mark.parametrize("fmt,m,n,k,k_block,s,mode,recipe", CHAIN_CASES)
def test_chained_run_sums_are_exact(fmt, m, n, k, k_block, s, mode, recipe):
    """The launch configuration ozaki_dgemm times (run formation on): the stored words are the exact sums of runs of
    consecutive pairs of one anti-diagonal; every run may only join pairs that carry the same power-of-two scale for
    that element, must stay inside the exact window of Eq. 11, and every pair must be covered exactly once."""
    A, B = _recipe(recipe, m, n, k, seed=m + 2 * n + k)
    Ad, Bd = _upload(A, B)
    plan, blocks = _oracle_products(A, B, fmt, s, k_block, mode)
    T, pairs = plan.num_blocks, oz.pair_order(s, mode)
    npairs = len(pairs)
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block, pair_set=PAIRS[mode])
    dt = torch.int32 if fmt == "int8" else torch.float32
    P = torch.full((T, npairs, n, m), -77, dtype=dt, device="cuda")
    L = torch.full((T, npairs, n, m), 99, dtype=torch.uint8, device="cuda")
    lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT[fmt], s, k_block, P, pair_set=PAIRS[mode], chained=1, run_len_out=L)
    assert lib.ozaki_last_device_status() == 0
    Pn, Ln = P.cpu().numpy(), L.cpu().numpy().astype(np.int64)
    window = formats.EXACT_WINDOW[fmt]
    longest = 0
    for t, br in enumerate(blocks):
        covered = np.zeros((npairs, n, m), dtype=np.int64)
        for z, (p, q) in enumerate(pairs):
            e_z = (br.c_a[p - 1][None, :] + br.c_b[q - 1][:, None])                      # (n, m) scale exponent of pair z
            run = Ln[t, z]
            want = np.zeros((n, m), dtype=np.int64)
            bound = np.zeros((n, m), dtype=np.int64)
            for j in range(int(run.max())):
                inside = run > j
                pj, qj = pairs[z + j] if z + j < npairs else (0, 0)
                assert not inside.any() or (pj + qj == p + q and pj == p + j), (t, z, j)     # same anti-diagonal, consecutive
                e_j = br.c_a[pj - 1][None, :] + br.c_b[qj - 1][:, None]
                assert np.array_equal(e_j[inside], e_z[inside]), (t, z, j)                # equal scale for the element
                want += np.where(inside, br.products[z + j].T, 0)
                bound += np.where(inside, plan.k_block << (2 * plan.b), 0)
                covered[z + j] += inside
            assert bound.max() <= window, (t, z)
            assert np.array_equal(Pn[t, z], _as_device_words(want.T, fmt, plan.b)), (t, z)
            longest = max(longest, int(run.max()))
        assert covered.min() == 1 and covered.max() == 1, t                                # every pair in exactly one run
    limit = max(1, min(32, window // (plan.k_block << (2 * plan.b))))
    assert longest <= limit
    if recipe in ("binade", "u110") and limit > 1:
        assert longest > 1                                                                  # runs do form on regular ladders
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
    ("int8", 300, 270, 520, 0, 10, 4.0),
    ("int8", 100, 600, 1000, 384, 9, 2.0),
    ("int8", 513, 255, 2048, 0, 9, 1.0),
]


def _run_dgemm(m, n, k, Ad, Bd, fmt, s, k_block, accum, mode="triangle", rule="runs", ldc=None, mem_cap=0, minimum=False):
    ldc = ldc or m
    Cd = torch.full((n, ldc), float("nan"), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block, pair_set=PAIRS[mode], minimum=minimum)
    lib.ozaki_dgemm_ex(m, n, k, Ad, m, Bd, k, Cd, ldc, FMT[fmt], s, k_block, ACC[accum], PAIRS[mode], SUM[rule], mem_cap)
    assert lib.ozaki_last_device_status() == 0
    ws.close()
    return Cd.cpu().numpy()


def _bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


@pytest.mark.parametrize("fmt,m,n,k,k_block,s,phi", DGEMM_CASES)
def test_dgemm_matches_oracle(fmt, m, n, k, k_block, s, phi):
    """All accumulation modes and rules of one problem: bit-identical to the oracle rule each implements; the default
    mode also against the PLAIN oracle (the paper's term-by-term FP64 sum): never a larger error against the exact
    product on 1024 and more entries, and at most a few units in the last place away."""
    A, B = inputs.phi_pair(m, n, k, phi, seed=7 * m + n + k)
    Ad, Bd = _upload(A, B)
    ldc = m + 3
    want = {rule: oz.ozaki_dgemm(A, B, fmt, s, k_block, accumulate=rule) for rule in oz.ACCUMULATE_RULES}
    got = {}
    for accum, rule in (("hw", "runs"), ("emu", "runs"), ("hw", "plain"), ("emu", "plain"), ("exact", "runs")):
        Cfull = _run_dgemm(m, n, k, Ad, Bd, fmt, s, k_block, accum, rule=rule, ldc=ldc)
        assert np.all(np.isnan(Cfull[:, m:]))                         # the padding of ldc is not touched
        C = Cfull[:, :m].T
        oracle_rule = "exact" if accum == "exact" else rule
        assert np.array_equal(_bits(C), _bits(want[oracle_rule])), (accum, rule)
        got[(accum, rule)] = C
    # the default mode against the plain oracle and the exact product
    C = got[("emu", "runs")]
    ent = exact.sample_entries(m, n, 1024, seed=m)
    ii, jj = np.array([e[0] for e in ent]), np.array([e[1] for e in ent])
    e_dev = exact.sampled_errors_fast(A, B, ent, C[ii, jj])[0]
    e_plain = exact.sampled_errors_fast(A, B, ent, want["plain"][ii, jj])[0]
    e_exact = exact.sampled_errors_fast(A, B, ent, got[("exact", "runs")][ii, jj])[0]
    ulps = int(exact.ulp_distance(C, want["plain"]).max())
    print(f"E_AB device(runs) {e_dev:.3e}  plain oracle {e_plain:.3e}  exact mode {e_exact:.3e}  max ulp distance to plain {ulps}")
    assert e_dev <= e_plain + 2.0 ** -53
    assert e_exact <= e_dev + 2.0 ** -53
    if s >= 7:
        assert e_dev <= BOUND(k) and e_plain <= BOUND(k)
    # a few entries the slow way (big integers), to keep the fast residuals honest on this very data
    few = ent[:6]
    slow = exact.sampled_errors(A, B, few, [C[i, j] for i, j in few])[2]
    fast = exact.sampled_errors_fast(A, B, few, [C[i, j] for i, j in few])[2]
    assert np.allclose(slow, fast, rtol=1e-6, atol=0)


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
        ("int8", inputs.uniform_1_10(20, 700, rng), 0),
        ("fp8", inputs.uniform_1_10(3, 50000, rng), 0),                          # a block longer than the register kernel takes
    ]
    for fmt, X, kb in cases:
        rows, k = X.shape
        want = oz.count_slices_to_exhaustion(X, fmt, kb)
        for is_B in (0, 1):
            Xd = torch.from_numpy(np.ascontiguousarray(X if is_B else X.T)).cuda()      # column-major k x rows / rows x k
            ws = device.Workspace(256 + 8 * rows * k + 256 + (12 * rows * (k + 64) + 256 if (kb or k) > 16384 else 0))
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
    C = _run_dgemm(40, 24, 96, Ad, Bd, "fp8", s, 0, "emu", mode="full").T
    assert np.array_equal(_bits(C), _bits(oz.ozaki_dgemm(A, B, "fp8", s, 0, mode="full", accumulate="runs")))
    Cx = _run_dgemm(40, 24, 96, Ad, Bd, "fp8", s, 0, "exact", mode="full").T
    for i in range(0, 40, 7):
        for j in range(0, 24, 5):
            ex = exact.exact_dot(A[i, :], B[:, j])
            assert abs(Fraction(float(C[i, j])) - ex) <= Fraction(float(np.spacing(abs(C[i, j])))) , (i, j)
            assert Cx[i, j] == exact.round_fraction_to_double(ex), (i, j)          # the exact mode: correctly rounded


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
@pytest.mark.parametrize("accum", ["hw", "emu", "exact"])
def test_all_pairs_mode_matches_oracle(fmt, m, n, k, k_block, s, phi, accum):
    """OZAKI_PAIRS_ALL: all s*s slice pairs (the paper's setting), anti-diagonals 2s ... 2."""
    A, B = inputs.phi_pair(m, n, k, phi, seed=m + 3 * n)
    Ad, Bd = _upload(A, B)
    C = _run_dgemm(m, n, k, Ad, Bd, fmt, s, k_block, accum, mode="full").T
    Cref, blocks = oz.ozaki_dgemm(A, B, fmt, s, k_block, mode="full", return_blocks=True, accumulate="exact" if accum == "exact" else "runs")
    assert np.array_equal(_bits(C), _bits(Cref))
    if accum == "hw":
        Cp = _run_dgemm(m, n, k, Ad, Bd, fmt, s, k_block, accum, mode="full", rule="plain").T
        assert np.array_equal(_bits(Cp), _bits(oz.ozaki_dgemm(A, B, fmt, s, k_block, mode="full")))
        T, npairs = len(blocks), s * s
        ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, k_block, pair_set=lib.PAIRS_ALL)
        P = torch.zeros((T, npairs, n, m), dtype=torch.float32, device="cuda")
        lib.ozaki_pair_products(m, n, k, Ad, m, Bd, k, FMT[fmt], s, k_block, P, pair_set=lib.PAIRS_ALL)
        torch.cuda.synchronize()
        Pn = P.cpu().numpy()
        b = oz.make_plan(k, fmt, k_block).b
        for t, br in enumerate(blocks):
            assert br.pairs == oz.pair_order(s, "full")
            for z, Pref in enumerate(br.products):
                assert np.array_equal(Pn[t, z], np.ldexp(Pref.astype(np.float64), -2 * b).astype(np.float32).T), (t, z)
        ws.close()


@pytest.mark.parametrize("fmt,m,n,k,k_block,s", [("fp8", 130, 90, 1024, 0, 11), ("fp6", 64, 70, 2048, 0, 11), ("int8", 130, 90, 1024, 0, 8),
                                                  ("fp16", 66, 130, 2048, 1024, 7)])
@pytest.mark.parametrize("accum", ["hw", "emu", "exact"])
def test_uniform_1_10_inputs_with_all_pairs_match_oracle(fmt, m, n, k, k_block, s, accum):
    """The paper's own workload (Section 5.1): entries uniform in (1, 10), every slice pair.  All first slices are
    positive, so the leading products are k times larger than a random-sign sum and tower over the sum of the less
    significant anti-diagonals: the case in which the integer-only running sum has to cut the sum down to the term's
    scale instead of bringing the term to the sum's."""
    rng = np.random.default_rng(m + n)
    A, B = inputs.uniform_1_10(m, k, rng), inputs.uniform_1_10(k, n, rng)
    Ad, Bd = _upload(A, B)
    C = _run_dgemm(m, n, k, Ad, Bd, fmt, s, k_block, accum, mode="full").T
    Cref = oz.ozaki_dgemm(A, B, fmt, s, k_block, mode="full", accumulate="exact" if accum == "exact" else "runs")
    assert np.array_equal(_bits(C), _bits(Cref))
    ent = [(i, j) for i in range(0, m, 7) for j in range(0, n, 5)]
    e_ab = exact.sampled_errors_fast(A, B, ent, [C[i, j] for i, j in ent])[0]
    assert e_ab <= 4 * k * 2.0 ** -53


def test_chunked_workspace_gives_identical_bits():
    """The smallest workspace processes the pairs in several passes with the block sum kept in work memory between
    them (one FP64 word per element, three words in the exact mode): same bits as with everything resident."""
    fmt, m, n, k, s = "fp8", 300, 270, 520, 8
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=5)
    Ad, Bd = _upload(A, B)
    for accum, rule in (("hw", "runs"), ("emu", "runs"), ("emu", "plain"), ("exact", "runs")):
        outs = [_run_dgemm(m, n, k, Ad, Bd, fmt, s, 0, accum, rule=rule, minimum=minimum) for minimum in (False, True, False)]
        assert np.array_equal(_bits(outs[0]), _bits(outs[1])) and np.array_equal(_bits(outs[0]), _bits(outs[2])), (accum, rule)
    for mode in ("triangle", "full"):
        a = _run_dgemm(m, n, k, Ad, Bd, fmt, 5, 128, "exact", mode=mode, minimum=True)
        b = _run_dgemm(m, n, k, Ad, Bd, fmt, 5, 128, "exact", mode=mode)
        assert np.array_equal(_bits(a), _bits(b))
        assert np.array_equal(_bits(a.T), _bits(oz.ozaki_dgemm(A, B, fmt, 5, 128, mode=mode, accumulate="exact")))


def test_two_contexts_with_their_own_streams_and_workspaces_run_side_by_side():
    """Calls of two contexts are interleaved from one host thread, each on its own stream with its own workspace, with
    no synchronisation between them: both results must be the ones of the contexts used alone."""
    probs = [("fp8", 600, 520, 1000, 384, 9, 2.0), ("fp16", 300, 270, 700, 256, 6, 1.0)]
    data, want = [], []
    for fmt, m, n, k, kb, s, phi in probs:
        A, B = inputs.phi_pair(m, n, k, phi, seed=m + k)
        data.append(_upload(A, B))
        want.append(oz.ozaki_dgemm(A, B, fmt, s, kb, accumulate="runs"))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [lib.ozaki_context_create(), lib.ozaki_context_create()]
    bufs, outs = [], []
    for c, st, (fmt, m, n, k, kb, s, phi) in zip(ctxs, streams, probs):
        lib.ozaki_context_use(c)
        nbytes = lib.ozaki_workspace_bytes(m, n, k, FMT[fmt], s, kb)
        bufs.append(torch.empty(nbytes, dtype=torch.uint8, device="cuda"))
        lib.ozaki_set_stream(st.cuda_stream)
        lib.ozaki_set_workspace(bufs[-1], nbytes)
        outs.append(torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda"))
    torch.cuda.synchronize()
    for rep in range(3):
        for c, (Ad, Bd), Cd, (fmt, m, n, k, kb, s, phi) in zip(ctxs, data, outs, probs):
            lib.ozaki_context_use(c)
            lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, kb, ACC["emu" if rep % 2 else "hw"])
    for c, Cd, w in zip(ctxs, outs, want):
        lib.ozaki_context_use(c)
        assert lib.ozaki_last_device_status() == 0
        assert np.array_equal(_bits(Cd.cpu().numpy().T), _bits(w))
        lib.ozaki_set_workspace(None, 0)
    lib.ozaki_context_use(None)
    for c in ctxs:
        lib.ozaki_context_destroy(c)
    # the default context is untouched by all this: it still has no workspace
    Ad, Bd = data[0]
    assert lib.ozaki_dgemm(600, 520, 1000, Ad, 600, Bd, 1000, outs[0], 600, 0, 9, 384, 0, check=False) == lib.STATUS_WORKSPACE


def test_memory_capped_call_works_in_panels_and_gives_the_same_bits():
    """Outer-product-wise blocking (Section 4.3): with a cap on the work memory the product is formed panel by panel
    (rows of A x columns of B); rows and columns are sliced independently, so C has the bits of the uncapped call."""
    fmt, m, n, k, kb, s = "fp8", 1100, 700, 900, 512, 9
    A, B = inputs.phi_pair(m, n, k, 2.0, seed=21)
    Ad, Bd = _upload(A, B)
    full = _run_dgemm(m, n, k, Ad, Bd, fmt, s, kb, "emu")
    assert np.array_equal(_bits(full.T), _bits(oz.ozaki_dgemm(A, B, fmt, s, kb, accumulate="runs")))
    need_all = lib.ozaki_workspace_min_bytes(m, n, k, FMT[fmt], s, kb)
    need_one = lib.ozaki_workspace_min_bytes(256, 256, k, FMT[fmt], s, kb)
    for cap in (need_all // 2, need_all // 5, need_one):
        assert cap < need_all
        got = _run_dgemm(m, n, k, Ad, Bd, fmt, s, kb, "emu", mem_cap=cap)
        assert np.array_equal(_bits(got), _bits(full)), cap
    got = _run_dgemm(m, n, k, Ad, Bd, fmt, s, kb, "exact", mode="full", mem_cap=need_all // 3)
    assert np.array_equal(_bits(got), _bits(_run_dgemm(m, n, k, Ad, Bd, fmt, s, kb, "exact", mode="full")))
    # a cap below one 256 x 256 panel cannot work
    Cd = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, kb)
    assert lib.ozaki_dgemm_ex(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, kb, 0, 0, 0, need_one // 2, check=False) == lib.STATUS_WORKSPACE
    ws.close()


@pytest.mark.parametrize("fmt,m,n,k,s,b", [("fp8", 70, 40, 65536, 11, 4), ("fp8", 33, 40, 131072, 12, 3), ("fp6", 20, 300, 100000, 13, 3),
                                           ("int8", 40, 33, 131072, 8, 6), ("fp16", 40, 20, 65536, 9, 4)])
def test_unblocked_inner_dimensions_beyond_the_register_kernel(fmt, m, n, k, s, b):
    """Table 2's last rows run as printed: k = 65536 (b = 4) and k = 131072 (b = 3) without inner blocking; the
    slicing then streams through the vectors with its state in work memory."""
    assert lib.ozaki_plan(k, FMT[fmt])[1] == b == oz.make_plan(k, fmt).b
    A, B = inputs.phi_pair(m, n, k, 1.0, seed=k % 1000 + m)
    Ad, Bd = _upload(A, B)
    for accum in ("hw", "exact"):
        C = _run_dgemm(m, n, k, Ad, Bd, fmt, s, 0, accum).T
        Cref = oz.ozaki_dgemm(A, B, fmt, s, 0, accumulate="exact" if accum == "exact" else "runs")
        assert np.array_equal(_bits(C), _bits(Cref)), accum
    ent = exact.sample_entries(m, n, 64, seed=1)
    assert exact.sampled_errors_fast(A, B, ent, [C[i, j] for i, j in ent])[0] <= BOUND(k)
    # every entry at the row maximum: each product is +-k * 4^b units, the edge of the exact window for 65536 and 4
    if fmt == "fp8" and k == 65536:
        A1, B1 = np.ones((m, k)), np.ones((k, n))
        B1[:, ::2] = -1.0
        A1d, B1d = _upload(A1, B1)
        assert np.array_equal(_run_dgemm(m, n, k, A1d, B1d, fmt, 2, 0, "emu").T, A1 @ B1)


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
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 33, 0, 0, check=False) == lib.STATUS_SLICE_COUNT
    assert lib.ozaki_dgemm_ex(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0, 2, 0, 0, check=False) == -14
    assert lib.ozaki_dgemm_ex(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 0, 0, 2, 0, check=False) == -15
    assert lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, 0, 4, 0, 3, check=False) == -13
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


FULL_SIZE_CASES = [
    # configuration, slice count (0: the calibrated full-accuracy count)
    ("c2_4096_fp8_hw", 0), ("c2_4096_fp8_hw", 4), ("c2_4096_fp8_hw", 10),      # config 2 sweeps the slice count
    ("c3_8192_fp8_emu", 0), ("c5a_16384x1024_fp8", 0), ("c5b_1024x65536_fp8", 0),
    ("c4_16384_fp16_kb1024", 0), ("c4_16384_fp16_kb4096", 0), ("c4_16384_fp8", 0),
]


@pytest.mark.parametrize("name,s_arg", FULL_SIZE_CASES)
def test_full_size_configs_on_sampled_rows_and_columns(name, s_arg):
    """At the benchmark's sizes the oracle cannot form all of C; rows of A and columns of B are sliced
    independently of each other, so the oracle run on a few rows and columns must reproduce exactly the
    corresponding entries of the device result (in the launch configuration bench.py times).  Beside the bits:
    the error against the exact product on 4096 entries, among them those of a 384 x 384 sample with the heaviest
    cancellation, next to the plain oracle's."""
    cfg = inputs.CONFIGS[name]
    m, n, k, fmt, kb = cfg["m"], cfg["n"], cfg["k"], cfg["fmt"], cfg["k_block"]
    s = s_arg or inputs.NUM_SLICES[name]
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
    assert np.array_equal(_bits(Csub), _bits(Cref))
    Cplain = oz.ozaki_dgemm(A[rows, :], B[:, cols], fmt, s, kb)
    all_ent = [(i, j) for i in range(ns) for j in range(ns)]
    e_dev = exact.sampled_errors_fast(A[rows, :], B[:, cols], all_ent, Csub.ravel())[0]
    e_plain = exact.sampled_errors_fast(A[rows, :], B[:, cols], all_ent, Cplain.ravel())[0]
    assert e_dev <= e_plain + 2.0 ** -53
    # 4096 entries against the exact product: from a 384 x 384 sample of C, the 2048 entries with the largest
    # (|A||B|) / |C| (most cancellation) and 2048 random ones
    big = 384 if k <= 16384 else 192
    r2 = np.sort(rng.choice(m, min(big, m), replace=False))
    c2 = np.sort(rng.choice(n, min(big, n), replace=False))
    Cs = Cd[torch.from_numpy(c2).cuda()][:, torch.from_numpy(r2).cuda()].cpu().numpy().T
    As, Bs = np.ascontiguousarray(A[r2, :]), np.ascontiguousarray(B[:, c2])
    ratio = (np.abs(As) @ np.abs(Bs)) / np.maximum(np.abs(Cs), 1e-300)
    worst = np.argsort(ratio, axis=None)[-2048:]
    rnd = rng.choice(Cs.size, 2048, replace=False)
    ent = [(int(f // Cs.shape[1]), int(f % Cs.shape[1])) for f in np.concatenate([worst, rnd])]
    e_ab, e_c, _, _ = exact.sampled_errors_fast(As, Bs, ent, [Cs[i, j] for i, j in ent])
    Cn = (torch.from_numpy(As).cuda() @ torch.from_numpy(Bs).cuda()).cpu().numpy()           # the GPU's native FP64 GEMM
    n_ab, n_c, _, _ = exact.sampled_errors_fast(As, Bs, ent, [Cn[i, j] for i, j in ent])
    print(f"  4096 entries: E_AB {e_ab:.3e} (native FP64 GEMM {n_ab:.3e}, bound {BOUND(k):.3e}), E_C {e_c:.3e} (native {n_c:.3e})", flush=True)
    if s >= inputs.S_BOUND[name]:
        assert e_ab <= BOUND(k)
    else:
        assert e_ab > BOUND(k)                        # too few slices must show (config 2's sweep starts at 4)
    if s == inputs.NUM_SLICES[name]:
        assert e_ab <= 4 * n_ab + 2.0 ** -53          # full accuracy: in the range of the native GEMM's error (calibrated on another sample)
    ws.close()
    del Cd, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["c3_8192_fp8_emu", "c4_16384_fp16_kb1024"])
def test_whole_slice_tiles_at_full_size(name):
    """Slices and exponents of whole 256-vector tiles -- the first, a middle and the last one of each operand --
    at the benchmark's size and in its launch configuration (the slicing kernel maps workgroups to vectors in an
    XCD-aware order that only shows at thousands of vectors)."""
    cfg = inputs.CONFIGS[name]
    m, n, k, fmt, kb = cfg["m"], cfg["n"], cfg["k"], cfg["fmt"], cfg["k_block"]
    s = inputs.NUM_SLICES[name]
    A, B, Ad, Bd = _config_inputs(cfg)
    plan = oz.make_plan(k, fmt, kb)
    T = plan.num_blocks
    for is_B, X, Xd, rows in ((0, A, Ad, m), (1, B.T, Bd, n)):
        ws = device.Workspace.for_problem(0 if is_B else rows, rows if is_B else 0, k, FMT[fmt], s, kb)
        dt = torch.int16 if fmt == "fp16" else torch.uint8
        slices = torch.empty(s * rows * k, dtype=dt, device="cuda")
        exps = torch.empty(T * s * rows, dtype=torch.int32, device="cuda")
        lib.ozaki_split(is_B, rows, k, Xd, k if is_B else rows, FMT[fmt], s, kb, slices, exps)
        assert lib.ozaki_last_device_status() == 0
        ws.close()
        sl = slices.view(T, s, rows, plan.k_block)                  # k is a multiple of the block length in these configurations
        ex = exps.view(T, s, rows)
        for first in (0, (rows // 512) * 256, rows - 256):
            sel = slice(first, first + 256)
            ref_codes, ref_exps, _ = oz.split_operand(np.ascontiguousarray(X[sel, :]), fmt, s, kb)
            got_c = sl[:, :, sel, :].cpu().numpy()
            got_e = ex[:, :, sel].cpu().numpy()
            if fmt == "fp16":
                got_c = got_c.view(np.uint16)
            for t in range(T):
                for p in range(s):
                    assert np.array_equal(got_e[t, p], ref_exps[t][p]), (is_B, first, t, p)
                    assert np.array_equal(got_c[t, p], ref_codes[t][p]), (is_B, first, t, p)
        del slices, exps, sl, ex
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
        fmt = ["fp8", "fp16", "fp6", "fp6_e3m2", "int8"][int(rng.integers(0, 5))]
        m, n = int(rng.integers(1, 400)), int(rng.integers(1, 400))
        k = int(rng.integers(1, 3000))
        kb = [0, int(rng.integers(1, k + 1)), int(rng.integers(1, 200))][int(rng.integers(0, 3))]
        s = int(rng.integers(1, 11))
        full = bool(rng.integers(0, 2)) and s <= 7
        phi = float(rng.choice([0.5, 1.0, 3.0]))
        accum, rule = [("hw", "runs"), ("emu", "runs"), ("exact", "runs"), ("hw", "plain"), ("emu", "plain")][int(rng.integers(0, 5))]
        cases.append((fmt, m, n, k, kb, s, full, phi, accum, rule))
    return cases


@pytest.mark.parametrize("fmt,m,n,k,kb,s,full,phi,accum,rule", _random_cases(40, seed=2025))
def test_random_shapes_and_parameters_match_oracle(fmt, m, n, k, kb, s, full, phi, accum, rule):
    """Seeded random problem shapes, block lengths (any value, also shorter than a chunk), slice counts, pair sets,
    formats, accumulation modes and rules: C bit-identical to the oracle rule the mode implements."""
    A, B = inputs.phi_pair(m, n, k, phi, seed=m * 7 + n * 3 + k)
    Ad, Bd = _upload(A, B)
    mode = "full" if full else "triangle"
    C = _run_dgemm(m, n, k, Ad, Bd, fmt, s, kb, accum, mode=mode, rule=rule).T
    Cref = oz.ozaki_dgemm(A, B, fmt, s, kb, mode=mode, accumulate="exact" if accum == "exact" else rule)
    assert np.array_equal(_bits(C), _bits(Cref))
