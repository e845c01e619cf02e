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
    assert set(seen) == set(inputs.CONFIGS) == set(inputs.NUM_SLICES) == set(inputs.S_BOUND)
    for name, (sb, sn) in seen.items():
        assert inputs.S_BOUND[name] == sb and inputs.NUM_SLICES[name] == sn, name
