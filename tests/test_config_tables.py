"""The slice counts hard-coded for the benchmark configurations are the calibrated ones."""
import os

from paper_2508_00441_amd import inputs


def test_num_slices_table_matches_calibration_file(golden_dir):
    seen = {}
    with open(os.path.join(golden_dir, "slices_per_config.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, s_bound, s_native = line.split()[:3]
            seen[name] = (int(s_bound), int(s_native))
    int8 = {name.split("@")[0]: v for name, v in seen.items() if name.endswith("@int8")}
    seen = {name: v for name, v in seen.items() if "@" not in name}
    assert set(seen) == set(inputs.CONFIGS) == set(inputs.NUM_SLICES) == set(inputs.S_BOUND)
    for name, (sb, sn) in seen.items():
        assert inputs.S_BOUND[name] == sb and inputs.NUM_SLICES[name] == sn, name
    # the same workloads with INT8 slices (lines "<config>@int8")
    assert set(int8) == set(inputs.NUM_SLICES_INT8)
    for name, (sb, sn) in int8.items():
        assert inputs.NUM_SLICES_INT8[name] == sn, name


def test_paper_workload_uses_the_slice_counts_of_table_2(golden_dir):
    """Section 5.1 workload: U(1,10) square matrices, all s^2 pairs, s^2 = the Table 2 entry for the block length."""
    table = {}
    with open(os.path.join(golden_dir, "table2_min_gemms.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            table[int(parts[0])] = parts[1:]
    for name, cfg in inputs.PAPER_CONFIGS.items():
        s = inputs.PAPER_NUM_SLICES[name]
        kb = cfg["k_block"] or cfg["k"]
        col = 0 if cfg["fmt"] == "fp16" else 2                  # FP16 / FP8 E4M3 with FP32 accumulation
        assert s * s == int(table[kb][col]), name
        assert cfg["pairs"] == "all" and cfg["dist"] == "u110" and cfg["m"] == cfg["n"] == cfg["k"]


def test_bench_refuses_more_than_one_gpu():
    """One GPU per box: the benchmark says so and exits instead of pretending to scale."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr and res.stdout.strip() == ""
