#!/usr/bin/env python3
"""Benchmark of the Ozaki-scheme DGEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--num-slices S] [--no-cpu-baseline]

One step = one full ozaki_dgemm call (slicing of A and B, all slice-pair GEMMs, FP64 accumulation and
rescale) on seeded synthetic inputs already resident in HBM; the workspace is allocated before the timed
region (as in the paper's Section 5.1).  Prints ONE JSON line:

  value            effective FP64 TFLOP/s = 2 m n k / time per step   (the paper's Section 5.4 unit)
  roofline         the slice-pair GEMM kernel against the dense FP8 / FP16 MFMA peak; `achieved` counts the
                   s(s+1)/2 slice GEMMs (2 m n k flop each) over the kernel time measured with HIP events
                   on the library's stream inside the timed region
  cpu_baseline     the CPU oracle timed on a bounded sample of the same workload (rows of A x columns of B
                   at the full inner dimension), in the same unit; the same leg checks the device result
                   bit for bit against the oracle on that sample and reports the error against the exact
                   big-integer product next to a native FP64 GEMM on the same entries
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"fp8": 5000.0, "fp16": 2500.0, "fp6": 10100.0}          # MI355X dense MFMA peaks
DTYPE_NAMES = {"fp8": "fp8_e4m3", "fp16": "fp16", "fp6": "fp6_e2m3"}
DEFAULT_CONFIG = "c3_8192_fp8_emu"                      # the configuration the metric is quoted on (n = 8192)
# L2-fill + write-back bytes of one pair_gemm_kernel launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (scaled by the 1 GiB copy-calibration kernel); see profiles/ozaki_dgemm_c3_8192_fp8_emu.md.  Only valid for
# the configuration's calibrated slice count.
MEASURED_TRAFFIC_BYTES = {("c3_8192_fp8_emu", "fp8"): 120.91 * 2 ** 30, ("c3_8192_fp8_emu", "fp6"): 90.21 * 2 ** 30}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default=DEFAULT_CONFIG)
    ap.add_argument("--num-slices", type=int, default=0, help="0: the calibrated full-accuracy count of the configuration")
    ap.add_argument("--accum", choices=["hw", "emu"], default=None, help="override the configuration's accumulation mode")
    ap.add_argument("--slice-format", choices=["fp8", "fp16", "fp6"], default=None,
                    help="override the configuration's slice format (fp6 = E2M3: same slices and same C as fp8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sample", type=int, default=0, help="rows/columns of the CPU-oracle sample (0: sized for ~15 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one elementwise FP32 pass over 1 GiB (reads 1 GiB, writes 1 GiB) before the timed "
                         "region, so that a counter run can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    return ap.parse_args()


def cpu_baseline_leg(cfg, s, A, B, Cd, sample):
    """Oracle on `sample` rows x `sample` columns at full k: timing, bit parity of the device result on that
    sample, and errors against the exact product (device, oracle and native FP64 GEMM on the GPU)."""
    import numpy as np
    import torch
    from oracle import exact, ozaki_oracle as oz

    m, n, k = cfg["m"], cfg["n"], cfg["k"]
    rng = np.random.default_rng(99)
    rows = np.sort(rng.choice(m, min(sample, m), replace=False))
    cols = np.sort(rng.choice(n, min(sample, n), replace=False))
    As, Bs = np.ascontiguousarray(A[rows, :]), np.ascontiguousarray(B[:, cols])
    t0 = time.perf_counter()
    Cref = oz.ozaki_dgemm(As, Bs, cfg["fmt"], s, cfg["k_block"], mode="full" if cfg.get("pairs") == "all" else "triangle", accumulate="runs")
    t_cpu = time.perf_counter() - t0
    Csub = Cd[torch.from_numpy(cols).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy().T
    bit_equal = bool(np.array_equal(Csub.view(np.uint64), Cref.view(np.uint64)))
    # errors against the exact product on a few entries of the sample
    ne = 32
    ii, jj = rng.integers(0, len(rows), ne), rng.integers(0, len(cols), ne)
    ent = [(int(i), int(j)) for i, j in zip(ii, jj)]
    dev = exact.sampled_errors(As, Bs, ent, [Csub[i, j] for i, j in ent])
    Ad = torch.from_numpy(np.ascontiguousarray(As)).cuda()
    Bd = torch.from_numpy(np.ascontiguousarray(Bs)).cuda()
    Cnat = (Ad @ Bd).cpu().numpy()                                     # native FP64 GEMM of the GPU (context)
    nat = exact.sampled_errors(As, Bs, ent, [Cnat[i, j] for i, j in ent])
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    flop = 2.0 * len(rows) * len(cols) * k
    return {
        "cpu_baseline": {
            "value": flop / t_cpu / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle ozaki_dgemm on {len(rows)} rows of A x {len(cols)} columns of B at full k={k}, "
                      f"s={s}, {t_cpu:.1f} s; value = 2*rows*cols*k/time",
        },
        "parity": {"device_equals_oracle_bitwise_on_sample": bit_equal, "sample_entries": int(Csub.size)},
        "max_rel_err": {
            "entries": ne, "bound_4k_2^-53": 4 * k * 2.0 ** -53,
            "ozaki_E_AB": dev[0], "ozaki_E_C": dev[1], "native_fp64_E_AB": nat[0], "native_fp64_E_C": nat[1],
        },
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "sharding over several GPUs is not implemented", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2508_00441_amd import binding as lib, device, inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    lib.load()
    cfg = dict(inputs.CONFIGS.get(args.config) or inputs.PAPER_CONFIGS[args.config])
    if args.accum:
        cfg["accum"] = args.accum
    if args.slice_format:
        cfg["fmt"] = args.slice_format
    m, n, k, fmt, kb = cfg["m"], cfg["n"], cfg["k"], cfg["fmt"], cfg["k_block"]
    s = args.num_slices or inputs.NUM_SLICES.get(args.config) or inputs.PAPER_NUM_SLICES[args.config]
    all_pairs = cfg.get("pairs") == "all"
    pairs = s * s if all_pairs else s * (s + 1) // 2
    pair_set = lib.PAIRS_ALL if all_pairs else lib.PAIRS_TRIANGLE
    fmt_id, acc_id = lib.SLICE_FORMATS[fmt], lib.ACCUM_MODES[cfg["accum"]]

    A, B = inputs.config_pair(cfg, seed=0)
    Ad, Bd = device.to_device_colmajor(A), device.to_device_colmajor(B)
    Cd = torch.empty((n, m), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, fmt_id, s, kb, pair_set=pair_set)

    def step():
        lib.ozaki_dgemm_ex(m, n, k, Ad, m, Bd, k, Cd, m, fmt_id, s, kb, acc_id, pair_set, lib.SUM_RUNS, 0)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    lib.ozaki_profile_enable(True)
    lib.ozaki_profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    phase_ms, launches = lib.ozaki_profile_read()
    lib.ozaki_profile_enable(False)
    assert lib.ozaki_last_device_status() == 0

    sec_per_step = (t1 - t0) / args.steps
    flop = 2.0 * m * n * k
    eff_tflops = flop / sec_per_step / 1e12
    gemm_launch_ms = phase_ms[1] / max(launches[1], 1)
    gemm_flop_per_launch = pairs * flop * args.steps / max(launches[1], 1)      # blocks x chunks launches share the pairs
    achieved = gemm_flop_per_launch / (gemm_launch_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[fmt]

    out = {
        "metric": "effective FP64 TFLOPS (2mnk/t) at n=8192; % FP8 MFMA peak; max rel err",
        "value": eff_tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAMES[fmt], "data": "synthetic",
        "config": {
            "workload": f"{args.config}: m={m} n={n} k={k}, entries "
                        + ("U(1,10)" if cfg.get("dist") == "u110" else f"(U(0,1)-0.5)*exp({cfg['phi']}*N(0,1))") + " seed 0",
            "slice_format": fmt, "num_slices": s, "slice_pairs": pairs, "k_block": kb or k,
            "accum_mode": "integer-emulated FP64" if cfg["accum"] == "emu" else "hardware FP64",
        },
        "roofline": {
            "kernel": "pair_gemm_kernel", "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
            "frac": achieved / peak,
            "traffic": MEASURED_TRAFFIC_BYTES.get((args.config, fmt)) if not args.num_slices else None, "traffic_unit": "bytes per launch",
            "avg_launch_ms": gemm_launch_ms, "launches_per_step": launches[1] / args.steps,
        },
        "phases_ms_per_step": {"slicing": phase_ms[0] / args.steps, "pair_gemms": phase_ms[1] / args.steps,
                               "accumulate_rescale": phase_ms[2] / args.steps},
        "mfma_frac_of_total_time": pairs * flop / sec_per_step / 1e12 / peak,
    }
    if not args.no_cpu_baseline:
        # context: the GPU's native FP64 GEMM on the same operands (C^T = B^T A^T in torch's row-major view)
        try:
            ref = torch.matmul(Bd, Ad)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for _ in range(3):
                ref = torch.matmul(Bd, Ad)
            torch.cuda.synchronize()
            out["native_fp64_dgemm_tflops"] = flop / ((time.perf_counter() - t2) / 3) / 1e12
            del ref
        except RuntimeError:                     # no room left beside the workspace
            out["native_fp64_dgemm_tflops"] = None
        sample = args.sample or {256: 256, 1024: 2048, 4096: 2048, 8192: 1536, 16384: 1280, 65536: 512}.get(k, 256)
        out.update(cpu_baseline_leg(cfg, s, A, B, Cd, sample))
    ws.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
