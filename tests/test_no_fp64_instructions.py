"""The integer-only accumulation kernels (emulated FP64 and the fixed-point mode) and the slicing kernels must contain
no FP64 instruction at all, and the hardware-FP64 accumulation kernel no FP64 multiply or fused multiply-add (the
product is formed on the matrix unit only).  Checked on the compiler's own assembly listing of the kernels (hipcc -S
cross-compiles without a GPU); a kernel's body runs from its label to its .Lfunc_end marker, so code behind an early
exit is inspected too."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_00441_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
F64 = r"\bv_\w*f64\w*"


def _kernel_bodies(src, tmp_path):
    from paper_2508_00441_amd import build
    out = tmp_path / (src + ".s")
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.check_call([HIPCC] + flags + ["--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", str(out)],
                          stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = out.read_text()
    bodies = {}
    for m in re.finditer(r"^(_Z\w+):[^\n]*\n(.*?)^\.Lfunc_end\d+:", text, flags=re.S | re.M):
        bodies[m.group(1)] = m.group(2)
    return bodies


def _only(bodies, fragment):
    hit = [b for n, b in bodies.items() if fragment in n]
    assert len(hit) == 1, (fragment, [n for n in bodies if fragment in n])
    assert hit[0].count("s_endpgm") >= 1
    return hit[0]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_integer_only_kernels_use_no_fp64(tmp_path):
    acc = _kernel_bodies("accumulate.hip", tmp_path)
    # accumulate_kernel<MODE, PINT>: MODE 0 hardware FP64, 1 emulated, 2 fixed point; PINT: INT32 products
    for pint in ("Lb0E", "Lb1E"):
        for mode in (1, 2):
            body = _only(acc, f"accumulate_kernelILi{mode}E{pint}")
            assert body.count("s_endpgm") >= 2                       # the early exit of a non-final pass and the normal one
            assert not re.search(F64, body), f"FP64 instruction in the integer-only accumulation kernel (mode {mode})"
        hw = _only(acc, f"accumulate_kernelILi0E{pint}")
        used = set(re.findall(r"\b(v_\w*f64\w*)", hw))
        assert used and all(re.match(r"v_(add|ldexp|cvt)_", u) for u in used), used      # adds, exponent scaling, converts only
    assert not re.search(F64, _only(acc, "axpby_kernelILb1E")), "FP64 instruction in the emulated scaling kernel"
    used = set(re.findall(r"\b(v_\w*f64\w*)", _only(acc, "axpby_kernelILb0E")))
    assert used and all(re.match(r"v_(add|mul)_f64", u) for u in used), used         # no fused multiply-add
    assert not re.search(F64, _only(acc, "add_emulated_kernel"))
    split = _kernel_bodies("split.hip", tmp_path)
    sk = [b for n, b in split.items() if "split_kernel" in n]
    assert len(sk) == 40              # 8 launch shapes x 5 slice formats
    stream = [b for n, b in split.items() if "split_stream_kernel" in n]
    assert len(stream) == 5
    for body in sk + stream:
        assert not re.search(F64, body), "FP64 instruction in a slicing kernel"
    gemm = _kernel_bodies("pair_gemm.hip", tmp_path)
    assert len(gemm) == 5
    for n, body in gemm.items():
        assert not re.search(F64, body)
        assert "v_mfma_f32_32x32x64_f8f6f4" in body or "v_mfma_f32_32x32x16_f16" in body or "v_mfma_i32_32x32x32_i8" in body
