"""Calibrates the number of slices per benchmark configuration with the CPU oracle only.

For each configuration a fixed sample of rows of A and columns of B (full inner dimension) is pushed
through the oracle for a range of slice counts s, and the result is compared with the exact big-integer
product on sampled entries:

  s_bound   smallest s whose max |C_hat - C*| / (|A||B|) is <= 4 k 2^-53   (the stated bound)
  s_native  smallest s whose error is <= that of a plain FP64 GEMM (numpy) on the same entries

Usage:  python tests/golden/calibrate_slices.py [config[@format] ...]      -> tests/golden/slices_per_config.txt
A name like c3_8192_fp8_emu@int8 calibrates the configuration with another slice format.  Lines of configurations that
are not named on the command line are kept.  Calls nothing but oracle/ and the input generators.
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import exact, ozaki_oracle as oz  # noqa: E402
from paper_2508_00441_amd import inputs  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "slices_per_config.txt")
NSAMPLE = 24          # rows and columns sampled
NENTRIES = 96         # entries compared with the exact product


def sample_operands(cfg):
    """Only the sampled rows/columns are generated at full size when the matrices are huge: the generator
    is called for the whole matrix (so the entries are those of the benchmark) and then sub-sampled."""
    A, B = inputs.phi_pair(cfg["m"], cfg["n"], cfg["k"], cfg["phi"], seed=0)
    rng = np.random.default_rng(2025)
    rows = np.sort(rng.choice(cfg["m"], NSAMPLE, replace=False))
    cols = np.sort(rng.choice(cfg["n"], NSAMPLE, replace=False))
    return np.ascontiguousarray(A[rows, :]), np.ascontiguousarray(B[:, cols])


def calibrate(name, cfg):
    if "@" in name:
        cfg = dict(cfg, fmt=name.split("@")[1])
    As, Bs = sample_operands(cfg)
    k = cfg["k"]
    rng = np.random.default_rng(7)
    ent = [(int(i), int(j)) for i, j in zip(rng.integers(0, NSAMPLE, NENTRIES), rng.integers(0, NSAMPLE, NENTRIES))]
    native = exact.sampled_errors(As, Bs, ent, [(As @ Bs)[i, j] for i, j in ent])
    bound = 4 * k * 2.0 ** -53
    rows = []
    s_bound = s_native = None
    for s in range(4, 33):
        C = oz.ozaki_dgemm(As, Bs, cfg["fmt"], s, cfg["k_block"], accumulate="runs")
        e_ab, e_c, _, _ = exact.sampled_errors(As, Bs, ent, [C[i, j] for i, j in ent])
        rows.append((s, e_ab, e_c))
        if s_bound is None and e_ab <= bound:
            s_bound = s
        if s_native is None and e_ab <= native[0]:
            s_native = s
        if s_bound is not None and s_native is not None and s >= s_native + 1:
            break
    return dict(name=name, s_bound=s_bound, s_native=s_native, bound=bound, native_e_ab=native[0], native_e_c=native[1], sweep=rows)


def main(argv):
    names = argv or list(inputs.CONFIGS)
    header = ["# Slices per benchmark configuration, calibrated with the CPU oracle against the exact big-integer product",
              f"# on {NENTRIES} entries of a {NSAMPLE} x {NSAMPLE} sample of rows/columns (written by calibrate_slices.py).",
              "# config  s_bound  s_native  bound(4k2^-53)  native_E_AB  native_E_C  | sweep s:E_AB ..."]
    kept = {}
    if os.path.exists(OUT):
        with open(OUT) as f:
            for line in f:
                if line.strip() and not line.startswith("#"):
                    kept[line.split()[0]] = line.rstrip("\n")
    for name in names:
        t0 = time.time()
        r = calibrate(name, inputs.CONFIGS[name.split("@")[0]])
        sweep = " ".join(f"{s}:{e:.2e}" for s, e, _ in r["sweep"])
        kept[name] = f"{name} {r['s_bound']} {r['s_native']} {r['bound']:.3e} {r['native_e_ab']:.3e} {r['native_e_c']:.3e} | {sweep}"
        print(kept[name], f"({time.time() - t0:.0f} s)", flush=True)
    with open(OUT, "w") as f:
        f.write("\n".join(header + list(kept.values())) + "\n")


if __name__ == "__main__":
    main(sys.argv[1:])
