"""The integer-emulated accumulation kernel and the slicing kernels must contain no FP64 instruction at all, and the
hardware-FP64 accumulation kernel no FP64 multiply or fused multiply-add (the product is formed on the matrix unit
only).  Checked on the compiler's own assembly listing of the kernels (hipcc -S cross-compiles without a GPU)."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_00441_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _kernel_bodies(src, tmp_path):
    from paper_2508_00441_amd import build
    out = tmp_path / (src + ".s")
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.check_call([HIPCC] + flags + ["--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", str(out)],
                          stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = out.read_text()
    bodies = {}
    for m in re.finditer(r"^(_Z\w+):.*?\n(.*?)\n\s*s_endpgm", text, flags=re.S | re.M):
        bodies[m.group(1)] = m.group(2)
    return bodies


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_emulated_accumulation_and_slicing_use_no_fp64(tmp_path):
    acc = _kernel_bodies("accumulate.hip", tmp_path)
    emu = [b for n, b in acc.items() if "accumulate_kernelILb1" in n]
    hw = [b for n, b in acc.items() if "accumulate_kernelILb0" in n]
    assert len(emu) == 1 and len(hw) == 1
    assert not re.search(r"\bv_\w*f64\w*", emu[0]), "FP64 instruction in the integer-emulated accumulation kernel"
    used = set(re.findall(r"\b(v_\w*f64\w*)", hw[0]))
    assert used and all(re.match(r"v_(add|ldexp|cvt)_", u) for u in used), used      # adds, exponent scaling, converts only
    axpby_emu = [b for n, b in acc.items() if "axpby_kernelILb1" in n]
    axpby_hw = [b for n, b in acc.items() if "axpby_kernelILb0" in n]
    assert len(axpby_emu) == 1 and not re.search(r"\bv_\w*f64\w*", axpby_emu[0]), "FP64 instruction in the emulated scaling kernel"
    used = set(re.findall(r"\b(v_\w*f64\w*)", axpby_hw[0]))
    assert used and all(re.match(r"v_(add|mul)_f64", u) for u in used), used         # no fused multiply-add
    add_emu = [b for n, b in acc.items() if "add_emulated_kernel" in n]
    assert len(add_emu) == 1 and not re.search(r"\bv_\w*f64\w*", add_emu[0])
    split = _kernel_bodies("split.hip", tmp_path)
    sk = [b for n, b in split.items() if "split_kernel" in n]
    assert len(sk) >= 28              # 7 launch shapes x 4 slice formats
    for body in sk:
        assert not re.search(r"\bv_\w*f64\w*", body), "FP64 instruction in a slicing kernel"
    gemm = _kernel_bodies("pair_gemm.hip", tmp_path)
    for n, body in gemm.items():
        assert not re.search(r"\bv_\w*f64\w*", body)
        assert "v_mfma_f32_32x32x64_f8f6f4" in body or "v_mfma_f32_32x32x16_f16" in body
