#!/usr/bin/env python3
"""Benchmark of the Ozaki-scheme DGEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--num-slices S] [--accum hw|emu|exact]
                    [--slice-format fp8|fp6|fp16|int8] [--no-cpu-baseline] [--no-other-configs]

One step = one full ozaki_dgemm call (slicing of A and B, all slice-pair GEMMs, FP64 accumulation and
rescale) on seeded synthetic inputs already resident in HBM; the workspace is allocated before the timed
region (as in the paper's Section 5.1).  Prints ONE JSON line:

  value            effective FP64 TFLOP/s = 2 m n k / mean time per step   (the paper's Section 5.4 unit); best and
                   median step times (HIP events around every step) are in `step_ms`
  roofline         the slice-pair GEMM kernel against the dense FP8 / FP6 / FP16 / INT8 MFMA peak; `achieved` counts
                   the slice GEMMs (2 m n k flop each) over the kernel time measured with HIP events on the library's
                   stream inside the timed region
  cpu_baseline     the CPU oracle timed on a bounded sample of the same workload (rows of A x columns of B
                   at the full inner dimension), in the same unit; the same leg checks the device result
                   bit for bit against the oracle on that sample and reports the error against the exact
                   product on 4096 entries next to a native FP64 GEMM on the same entries
  other_configs    short runs of the other benchmark configurations (the small case, the 4096^3 slice-count sweep, the
                   two rectangular cases, the 16384^3 FP8 / k-blocked FP16 comparison, and the metric workload with FP6
                   and INT8 slices): time, effective TFLOP/s, GEMM fraction of peak, bit parity with the oracle on a sample
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"fp8": 5000.0, "fp16": 2500.0, "fp6": 10100.0, "int8": 5000.0}          # MI355X dense MFMA peaks (INT8: TOP/s)
DTYPE_NAMES = {"fp8": "fp8_e4m3", "fp16": "fp16", "fp6": "fp6_e2m3", "int8": "int8"}
DEFAULT_CONFIG = "c3_8192_fp8_emu"                      # the configuration the metric is quoted on (n = 8192)
# HBM-side bytes of one pair_gemm_kernel launch (L2 fills + write-backs) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/ (scaled by the 1 GiB copy-calibration pass); valid for the calibrated slice count only.
PROFILED_TRAFFIC = {}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "pair_gemm_traffic.json")
if os.path.exists(TRAFFIC_FILE):
    with open(TRAFFIC_FILE) as _f:
        PROFILED_TRAFFIC = json.load(_f)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default=DEFAULT_CONFIG)
    ap.add_argument("--num-slices", type=int, default=0, help="0: the calibrated full-accuracy count of the configuration")
    ap.add_argument("--accum", choices=["hw", "emu", "exact"], default=None, help="override the configuration's accumulation mode")
    ap.add_argument("--slice-format", choices=["fp8", "fp16", "fp6", "int8"], default=None,
                    help="override the configuration's slice format (fp6 = E2M3: same slices and same C as fp8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--sample", type=int, default=0, help="rows/columns of the CPU-oracle sample (0: sized for ~15 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one elementwise FP32 pass over 1 GiB (reads 1 GiB, writes 1 GiB) before the timed "
                         "region, so that a counter run can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    return ap.parse_args()


def oracle_rule(accum):
    return "exact" if accum == "exact" else "runs"


def cpu_baseline_leg(cfg, s, A, B, Cd, sample):
    """Oracle on `sample` rows x `sample` columns at full k: timing, bit parity of the device result on that
    sample, and errors against the exact product (device, plain oracle and native FP64 GEMM on the GPU)."""
    import numpy as np
    import torch
    from oracle import exact, ozaki_oracle as oz

    m, n, k = cfg["m"], cfg["n"], cfg["k"]
    rng = np.random.default_rng(99)
    rows = np.sort(rng.choice(m, min(sample, m), replace=False))
    cols = np.sort(rng.choice(n, min(sample, n), replace=False))
    As, Bs = np.ascontiguousarray(A[rows, :]), np.ascontiguousarray(B[:, cols])
    mode = "full" if cfg.get("pairs") == "all" else "triangle"
    t0 = time.perf_counter()
    Cref = oz.ozaki_dgemm(As, Bs, cfg["fmt"], s, cfg["k_block"], mode=mode, accumulate=oracle_rule(cfg["accum"]))
    t_cpu = time.perf_counter() - t0
    Csub = Cd[torch.from_numpy(cols).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy().T
    bit_equal = bool(np.array_equal(Csub.view(np.uint64), Cref.view(np.uint64)))
    # errors against the exact product: the 2048 entries of the sample with the most cancellation and 2048 random ones
    ratio = (np.abs(As) @ np.abs(Bs)) / np.maximum(np.abs(Csub), 1e-300)
    pick = np.concatenate([np.argsort(ratio, axis=None)[-2048:], rng.choice(Csub.size, min(2048, Csub.size), replace=False)])
    ent = [(int(f // Csub.shape[1]), int(f % Csub.shape[1])) for f in pick]
    dev = exact.sampled_errors_fast(As, Bs, ent, [Csub[i, j] for i, j in ent])
    Ad = torch.from_numpy(np.ascontiguousarray(As)).cuda()
    Bd = torch.from_numpy(np.ascontiguousarray(Bs)).cuda()
    Cnat = (Ad @ Bd).cpu().numpy()                                     # native FP64 GEMM of the GPU (context)
    nat = exact.sampled_errors_fast(As, Bs, ent, [Cnat[i, j] for i, j in ent])
    # the paper-plain accumulation rule (term-by-term FP64 sum of Eq. 10) on a smaller part of the sample
    sub = min(256, len(rows), len(cols))
    Cplain = oz.ozaki_dgemm(As[:sub], Bs[:, :sub], cfg["fmt"], s, cfg["k_block"], mode=mode)
    ent2 = [(i, j) for i in range(0, sub, 4) for j in range(0, sub, 4)]
    pl = exact.sampled_errors_fast(As[:sub], Bs[:, :sub], ent2, [Cplain[i, j] for i, j in ent2])
    dv2 = exact.sampled_errors_fast(As[:sub], Bs[:, :sub], ent2, [Csub[i, j] for i, j in ent2])
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
        "parity": {"device_equals_oracle_bitwise_on_sample": bit_equal, "sample_entries": int(Csub.size),
                   "oracle_rule": oracle_rule(cfg["accum"]),
                   "vs_plain_oracle": {"entries": len(ent2), "device_E_AB": dv2[0], "plain_oracle_E_AB": pl[0],
                                       "max_ulp_distance": int(exact.ulp_distance(Csub[:sub, :sub], Cplain).max())}},
        "max_rel_err": {
            "entries": len(ent), "bound_4k_2^-53": 4 * k * 2.0 ** -53,
            "ozaki_E_AB": dev[0], "ozaki_E_C": dev[1], "native_fp64_E_AB": nat[0], "native_fp64_E_C": nat[1],
        },
    }


class Runner:
    """Device operands, output and workspace of one configuration; `step()` is one full ozaki_dgemm call."""

    def __init__(self, name, cfg, s, inputs_cache=None):
        import torch
        from paper_2508_00441_amd import binding as lib, device, inputs
        self.lib, self.name, self.cfg, self.s = lib, name, cfg, s
        m, n, k = cfg["m"], cfg["n"], cfg["k"]
        key = (m, n, k, cfg.get("phi"), cfg.get("dist"))
        if inputs_cache is not None and key in inputs_cache:
            self.A, self.B, self.Ad, self.Bd = inputs_cache[key]
        else:
            self.A, self.B = inputs.config_pair(cfg, seed=0)
            self.Ad, self.Bd = device.to_device_colmajor(self.A), device.to_device_colmajor(self.B)
            if inputs_cache is not None:
                inputs_cache[key] = (self.A, self.B, self.Ad, self.Bd)
        self.all_pairs = cfg.get("pairs") == "all"
        self.pairs = s * s if self.all_pairs else s * (s + 1) // 2
        self.pair_set = lib.PAIRS_ALL if self.all_pairs else lib.PAIRS_TRIANGLE
        self.fmt_id, self.acc_id = lib.SLICE_FORMATS[cfg["fmt"]], lib.ACCUM_MODES[cfg["accum"]]
        self.Cd = torch.empty((n, m), dtype=torch.float64, device="cuda")
        self.ws = device.Workspace.for_problem(m, n, k, self.fmt_id, s, cfg["k_block"], pair_set=self.pair_set)

    def step(self):
        c = self.cfg
        self.lib.ozaki_dgemm_ex(c["m"], c["n"], c["k"], self.Ad, c["m"], self.Bd, c["k"], self.Cd, c["m"], self.fmt_id, self.s,
                                c["k_block"], self.acc_id, self.pair_set, self.lib.SUM_RUNS, 0)

    def timed(self, steps, warmup):
        """(mean seconds per step over the bracketed region, per-step ms list, phase ms, launches)"""
        import torch
        lib = self.lib
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        lib.ozaki_profile_enable(True)
        lib.ozaki_profile_read()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            self.step()
            marks[i + 1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        phase_ms, launches = lib.ozaki_profile_read()
        lib.ozaki_profile_enable(False)
        assert lib.ozaki_last_device_status() == 0
        per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
        return (t1 - t0) / steps, per_step, phase_ms, launches

    def close(self):
        self.ws.close()
        self.Cd = None


def short_run(name, cfg, s, cache, steps=5, sample=48):
    """One line of `other_configs`: timing plus bit parity with the oracle on sample x sample entries."""
    import numpy as np
    import torch
    from oracle import ozaki_oracle as oz
    r = Runner(name, cfg, s, cache)
    sec, per_step, phase_ms, launches = r.timed(steps, 2)
    m, n, k, fmt = cfg["m"], cfg["n"], cfg["k"], cfg["fmt"]
    flop = 2.0 * m * n * k
    rng = np.random.default_rng(7)
    rows = np.sort(rng.choice(m, min(sample, m), replace=False))
    cols = np.sort(rng.choice(n, min(sample, n), replace=False))
    Csub = r.Cd[torch.from_numpy(cols).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy().T
    Cref = oz.ozaki_dgemm(r.A[rows, :], r.B[:, cols], fmt, s, cfg["k_block"], mode="full" if r.all_pairs else "triangle",
                          accumulate=oracle_rule(cfg["accum"]))
    gemm_ms = phase_ms[1] / steps
    out = {"config": name, "slice_format": fmt, "num_slices": s, "slice_pairs": r.pairs, "k_block": cfg["k_block"] or k,
           "accum_mode": cfg["accum"], "ms_best": min(per_step), "ms_median": statistics.median(per_step),
           "eff_tflops": flop / (statistics.median(per_step) * 1e-3) / 1e12,
           "gemm_frac_of_peak": r.pairs * flop / (gemm_ms * 1e-3) / 1e12 / PEAK_TFLOPS[fmt],
           "phases_ms": [phase_ms[0] / steps, gemm_ms, phase_ms[2] / steps],
           "bits_equal_oracle_on_sample": bool(np.array_equal(Csub.view(np.uint64), Cref.view(np.uint64)))}
    r.close()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "sharding over several GPUs is not implemented", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2508_00441_amd import binding as lib, inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    lib.load()
    cfg = dict(inputs.CONFIGS.get(args.config) or inputs.PAPER_CONFIGS[args.config])
    if args.accum:
        cfg["accum"] = args.accum
    if args.slice_format:
        cfg["fmt"] = args.slice_format
    m, n, k, fmt, kb = cfg["m"], cfg["n"], cfg["k"], cfg["fmt"], cfg["k_block"]
    if args.num_slices:
        s = args.num_slices
    elif fmt == "int8" and args.config in inputs.NUM_SLICES_INT8:
        s = inputs.NUM_SLICES_INT8[args.config]
    else:
        s = inputs.NUM_SLICES.get(args.config) or inputs.PAPER_NUM_SLICES[args.config]
    cache = {}
    run = Runner(args.config, cfg, s, cache)
    pairs = run.pairs

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    sec_per_step, per_step, phase_ms, launches = run.timed(args.steps, args.warmup)

    flop = 2.0 * m * n * k
    eff_tflops = flop / sec_per_step / 1e12
    gemm_launch_ms = phase_ms[1] / max(launches[1], 1)
    gemm_flop_per_launch = pairs * flop * args.steps / max(launches[1], 1)      # blocks x chunks launches share the pairs
    achieved = gemm_flop_per_launch / (gemm_launch_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[fmt]
    traffic = PROFILED_TRAFFIC.get(f"{args.config}:{fmt}:{s}") if not args.accum else None

    out = {
        "metric": "effective FP64 TFLOPS (2mnk/t) at n=8192; % FP8 MFMA peak; max rel err",
        "value": eff_tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAMES[fmt], "data": "synthetic",
        "config": {
            "workload": f"{args.config}: m={m} n={n} k={k}, entries "
                        + ("U(1,10)" if cfg.get("dist") == "u110" else f"(U(0,1)-0.5)*exp({cfg['phi']}*N(0,1))") + " seed 0",
            "slice_format": fmt, "num_slices": s, "slice_pairs": pairs, "k_block": kb or k,
            "accum_mode": {"emu": "integer-emulated FP64", "hw": "hardware FP64", "exact": "192-bit fixed point, rounded once"}[cfg["accum"]],
        },
        "step_ms": {"best": min(per_step), "median": statistics.median(per_step), "mean": sec_per_step * 1e3,
                    "eff_tflops_at_best": flop / (min(per_step) * 1e-3) / 1e12},
        "roofline": {
            "kernel": "pair_gemm_kernel", "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
            "frac": achieved / peak,
            "traffic": traffic["bytes_per_launch"] if traffic else None, "traffic_unit": "bytes per launch",
            "traffic_source": traffic["source"] if traffic else None,
            "avg_launch_ms": gemm_launch_ms, "launches_per_step": launches[1] / args.steps,
        },
        "phases_ms_per_step": {"slicing": phase_ms[0] / args.steps, "pair_gemms": phase_ms[1] / args.steps,
                               "accumulate_rescale": phase_ms[2] / args.steps},
        "mfma_frac_of_total_time": pairs * flop / sec_per_step / 1e12 / peak,
    }
    if not args.no_cpu_baseline:
        # context: the GPU's native FP64 GEMM on the same operands (C^T = B^T A^T in torch's row-major view)
        try:
            ref = torch.matmul(run.Bd, run.Ad)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for _ in range(3):
                ref = torch.matmul(run.Bd, run.Ad)
            torch.cuda.synchronize()
            out["native_fp64_dgemm_tflops"] = flop / ((time.perf_counter() - t2) / 3) / 1e12
            del ref
        except RuntimeError:                     # no room left beside the workspace
            out["native_fp64_dgemm_tflops"] = None
        sample = args.sample or {256: 256, 1024: 2048, 4096: 2048, 8192: 1536, 16384: 1280, 65536: 512}.get(k, 256)
        out.update(cpu_baseline_leg(cfg, s, run.A, run.B, run.Cd, sample))
    run.close()
    if not args.no_other_configs and args.config == DEFAULT_CONFIG and not (args.accum or args.slice_format or args.num_slices):
        others = []
        # the metric workload with the other slice formats of the same width class (same A and B, already resident)
        for f in ("fp6", "int8"):
            c2 = dict(cfg, fmt=f)
            others.append(short_run(args.config, c2, inputs.NUM_SLICES_INT8[args.config] if f == "int8" else s, cache, steps=3))
        cache.clear()
        torch.cuda.empty_cache()
        for name in ("c1_256_fp8_hw", "c5a_16384x1024_fp8", "c5b_1024x65536_fp8"):
            others.append(short_run(name, dict(inputs.CONFIGS[name]), inputs.NUM_SLICES[name], cache))
            cache.clear()
            torch.cuda.empty_cache()
        c2cfg = dict(inputs.CONFIGS["c2_4096_fp8_hw"])
        for s2 in range(4, inputs.NUM_SLICES["c2_4096_fp8_hw"] + 1):
            others.append(short_run("c2_4096_fp8_hw", c2cfg, s2, cache, steps=3, sample=32))
        cache.clear()
        torch.cuda.empty_cache()
        # the 16384^3 comparison of unblocked FP8 with k-blocked FP16 slices (one pair of inputs serves the three)
        for name in ("c4_16384_fp8", "c4_16384_fp16_kb4096", "c4_16384_fp16_kb1024"):
            others.append(short_run(name, dict(inputs.CONFIGS[name]), inputs.NUM_SLICES[name], cache, steps=2, sample=32))
        cache.clear()
        out["other_configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
