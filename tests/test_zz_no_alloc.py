"""ozaki_dgemm_static, the entry point that allocates nothing (its work memory is a fixed array inside the library's
device code), against ozaki_dgemm with a caller workspace: same bits in C, on two calls in a row, the second with a
smaller input (the array then still holds what the first call left), and the size limit is an error, not a fault."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2508_00441_amd import binding as lib, device, inputs  # noqa: E402

FMT = lib.SLICE_FORMATS
ACC = lib.ACCUM_MODES


def _reference(m, n, k, Ad, Bd, fmt, s, kb, accum):
    """C of the existing entry point (caller workspace)."""
    Cd = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda")
    ws = device.Workspace.for_problem(m, n, k, FMT[fmt], s, kb)
    lib.ozaki_dgemm(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, kb, ACC[accum])
    assert lib.ozaki_last_device_status() == 0
    ws.close()
    return Cd.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib.load()
    lib.ozaki_set_workspace(None, 0)                                  # no caller workspace is set
    lib.ozaki_set_stream(torch.cuda.current_stream().cuda_stream)
    # first a problem that fills most of the array (several tiles, ragged edges, k-blocked), then a smaller one
    calls = [("fp8", 600, 520, 1000, 384, 11, 2.0, "emu"), ("fp8", 256, 256, 256, 0, 12, 0.5, "hw"),
             ("fp16", 130, 70, 300, 128, 6, 1.0, "emu"), ("fp6", 300, 270, 520, 0, 9, 4.0, "hw")]
    for fmt, m, n, k, kb, s, phi, accum in calls:
        need = lib.ozaki_workspace_min_bytes(m, n, k, FMT[fmt], s, kb)
        assert 0 < need <= lib.STATIC_SCRATCH_BYTES, (need, lib.STATIC_SCRATCH_BYTES)
        print(f"static-scratch call: fmt={fmt} m={m} n={n} k={k} k_block={kb} s={s} accum={accum} needs {need} bytes", flush=True)
        A, B = inputs.phi_pair(m, n, k, phi, seed=m + n + k)
        Ad, Bd = device.to_device_colmajor(A), device.to_device_colmajor(B)
        Cd = torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda")
        lib.ozaki_dgemm_static(m, n, k, Ad, m, Bd, k, Cd, m, FMT[fmt], s, kb, ACC[accum])
        assert lib.ozaki_last_device_status() == 0
        got = Cd.cpu().numpy()
        want = _reference(m, n, k, Ad, Bd, fmt, s, kb, accum)
        assert np.array_equal(got.view(np.uint64), want.view(np.uint64)), (fmt, m, n, k)
    # beyond the array: a clear error before anything is launched, and C is untouched
    m = n = k = 2048
    assert lib.ozaki_workspace_min_bytes(m, n, k, FMT["fp8"], 13, 0) > lib.STATIC_SCRATCH_BYTES
    Cd = torch.full((4,), 7.0, dtype=torch.float64, device="cuda")
    st = lib.ozaki_dgemm_static(m, n, k, Cd, m, Cd, k, Cd, m, FMT["fp8"], 13, 0, ACC["hw"], check=False)
    assert st == lib.STATUS_STATIC_LIMIT and "static" in lib.status_string(st)
    torch.cuda.synchronize()
    assert float(Cd.min()) == 7.0
    # a non-finite input is reported through the same status call
    A, B = inputs.phi_pair(64, 48, 96, 1.0, seed=3)
    A[5, 7] = np.nan
    Ad, Bd = device.to_device_colmajor(A), device.to_device_colmajor(B)
    Cd = torch.empty((48, 64), dtype=torch.float64, device="cuda")
    lib.ozaki_dgemm_static(64, 48, 96, Ad, 64, Bd, 96, Cd, 64, FMT["fp8"], 4, 0, ACC["hw"])
    assert lib.ozaki_last_device_status() == lib.STATUS_NONFINITE
    assert lib.ozaki_last_device_status() == 0
