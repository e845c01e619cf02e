"""ctypes binding of libozaki.so: the same entry points as include/ozaki_dgemm.h, argument marshalling only.

Every step of the Ozaki-scheme DGEMM runs in the HIP library; nothing here computes.  There is no CPU
fallback: loading fails loudly if the library has not been built (python -m paper_2508_00441_amd.build).

Device pointers may be given as torch CUDA tensors (their data_ptr() is passed) or as integers.
"""
from __future__ import annotations

import ctypes
import os
from typing import Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libozaki.so")

SLICE_FP8_E4M3 = 0
SLICE_FP16 = 1
SLICE_FP6_E2M3 = 2
SLICE_FP6_E3M2 = 3
SLICE_INT8 = 4
ACCUM_FP64_HW = 0
ACCUM_FP64_INT_EMU = 1
ACCUM_EXACT_FIXED = 2
PAIRS_TRIANGLE, PAIRS_ALL = 0, 1
SUM_RUNS, SUM_PLAIN = 0, 1
STATUS_OK, STATUS_INFEASIBLE, STATUS_WORKSPACE, STATUS_HIP_ERROR, STATUS_NONFINITE, STATUS_STATIC_LIMIT, STATUS_SLICE_COUNT = 0, 1, 3, 4, 5, 6, 7
STATIC_SCRATCH_BYTES = 64 << 20
MAX_SLICES = 32

SLICE_FORMATS = {"fp8": SLICE_FP8_E4M3, "fp16": SLICE_FP16, "fp6": SLICE_FP6_E2M3, "fp6_e3m2": SLICE_FP6_E3M2, "int8": SLICE_INT8}
ACCUM_MODES = {"hw": ACCUM_FP64_HW, "emu": ACCUM_FP64_INT_EMU, "exact": ACCUM_EXACT_FIXED}
PAIR_SETS = {"triangle": PAIRS_TRIANGLE, "full": PAIRS_ALL}
SUM_RULES = {"runs": SUM_RUNS, "plain": SUM_PLAIN}

#: every symbol include/ozaki_dgemm.h declares: name -> (restype, argtypes)
_i64, _int, _vp, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
SIGNATURES = {
    "ozaki_plan": (_int, [_i64, _int, ctypes.POINTER(_int), ctypes.POINTER(_int)]),
    "ozaki_dgemm": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _int, _i64, _int]),
    "ozaki_dgemm_ex": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _int, _i64, _int, _int, _int, _sz]),
    "ozaki_context_create": (_int, [ctypes.POINTER(_vp)]),
    "ozaki_context_destroy": (_int, [_vp]),
    "ozaki_context_use": (_int, [_vp]),
    "ozaki_workspace_bytes_ex": (_sz, [_i64, _i64, _i64, _int, _int, _i64, _int, _int]),
    "ozaki_dgemm_static": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _int, _i64, _int]),
    "ozaki_dgemm_scaled": (_int, [_i64, _i64, _i64, ctypes.c_double, _vp, _i64, _vp, _i64, ctypes.c_double, _vp, _i64, _int, _int,
                                  _i64, _int]),
    "ozaki_workspace_bytes_scaled": (_sz, [_i64, _i64, _i64, _int, _int, _i64]),
    "ozaki_count_slices": (_int, [_int, _i64, _i64, _vp, _i64, _int, _i64, ctypes.POINTER(ctypes.c_int)]),
    "ozaki_suggest_k_block": (_i64, [_i64, _int]),
    "ozaki_set_stream": (_int, [_vp]),
    "ozaki_workspace_bytes": (_sz, [_i64, _i64, _i64, _int, _int, _i64]),
    "ozaki_workspace_min_bytes": (_sz, [_i64, _i64, _i64, _int, _int, _i64]),
    "ozaki_set_workspace": (_int, [_vp, _sz]),
    "ozaki_last_device_status": (_int, []),
    "ozaki_last_hip_error": (_int, []),
    "ozaki_status_string": (ctypes.c_char_p, [_int]),
    "ozaki_profile_enable": (_int, [_int]),
    "ozaki_profile_read": (_int, [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(_int)]),
    "ozaki_split": (_int, [_int, _i64, _i64, _vp, _i64, _int, _int, _i64, _vp, _vp]),
    "ozaki_pair_products": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _int, _int, _i64, _int, _int, _vp, _vp]),
    "ozaki_fp64_add_emulated": (_int, [_vp, _vp, _vp, _i64]),
}

_lib = None


class OzakiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def load() -> ctypes.CDLL:
    """Loads libozaki.so once; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2508_00441_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _ptr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _check(status: int, where: str) -> int:
    if status != 0:
        raise OzakiError(status, where)
    return status


def status_string(status: int) -> str:
    return load().ozaki_status_string(status).decode()


def ozaki_plan(k_block: int, slice_format: int) -> Tuple[int, int]:
    """(rho, b) of Eq. 1-3 for one block length; host only."""
    rho, b = ctypes.c_int(0), ctypes.c_int(0)
    _check(load().ozaki_plan(k_block, slice_format, ctypes.byref(rho), ctypes.byref(b)), "ozaki_plan")
    return rho.value, b.value


def ozaki_set_stream(stream_handle: int) -> None:
    _check(load().ozaki_set_stream(stream_handle), "ozaki_set_stream")


def ozaki_suggest_k_block(k, slice_format) -> int:
    r = int(load().ozaki_suggest_k_block(k, slice_format))
    if r < 0:
        raise OzakiError(r, "ozaki_suggest_k_block")
    return r


def ozaki_context_create() -> int:
    """A new context (its handle as an integer); select it with ozaki_context_use."""
    h = _vp(None)
    _check(load().ozaki_context_create(ctypes.byref(h)), "ozaki_context_create")
    return int(h.value)


def ozaki_context_destroy(handle: int) -> None:
    _check(load().ozaki_context_destroy(handle), "ozaki_context_destroy")


def ozaki_context_use(handle) -> None:
    """Makes `handle` (None: the default context) the calling thread's current context."""
    _check(load().ozaki_context_use(handle), "ozaki_context_use")


def ozaki_workspace_bytes_ex(m, n, k, slice_format, num_slices, k_block, pair_set, minimum) -> int:
    return int(load().ozaki_workspace_bytes_ex(m, n, k, slice_format, num_slices, k_block, pair_set, 1 if minimum else 0))


def ozaki_workspace_bytes(m, n, k, slice_format, num_slices, k_block) -> int:
    return int(load().ozaki_workspace_bytes(m, n, k, slice_format, num_slices, k_block))


def ozaki_workspace_bytes_scaled(m, n, k, slice_format, num_slices, k_block) -> int:
    return int(load().ozaki_workspace_bytes_scaled(m, n, k, slice_format, num_slices, k_block))


def ozaki_workspace_min_bytes(m, n, k, slice_format, num_slices, k_block) -> int:
    return int(load().ozaki_workspace_min_bytes(m, n, k, slice_format, num_slices, k_block))


def ozaki_set_workspace(buf, nbytes: int) -> None:
    _check(load().ozaki_set_workspace(_ptr(buf), nbytes), "ozaki_set_workspace")


def ozaki_last_device_status() -> int:
    return int(load().ozaki_last_device_status())


def ozaki_last_hip_error() -> int:
    return int(load().ozaki_last_hip_error())


def ozaki_profile_enable(on: bool) -> None:
    _check(load().ozaki_profile_enable(1 if on else 0), "ozaki_profile_enable")


def ozaki_profile_read():
    """([ms_split, ms_gemm, ms_accumulate], [launches...]) accumulated since the last read."""
    ms = (ctypes.c_float * 3)()
    cnt = (ctypes.c_int * 3)()
    _check(load().ozaki_profile_read(ms, cnt), "ozaki_profile_read")
    return list(ms), list(cnt)


def ozaki_dgemm(m, n, k, A, lda, B, ldb, C, ldc, slice_format, num_slices, k_block, accum_mode, check: bool = True) -> int:
    st = load().ozaki_dgemm(m, n, k, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, slice_format, num_slices, k_block, accum_mode)
    return _check(st, "ozaki_dgemm") if check else st


def ozaki_dgemm_ex(m, n, k, A, lda, B, ldb, C, ldc, slice_format, num_slices, k_block, accum_mode, pair_set=PAIRS_TRIANGLE,
                   sum_rule=SUM_RUNS, mem_cap=0, check: bool = True) -> int:
    st = load().ozaki_dgemm_ex(m, n, k, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, slice_format, num_slices, k_block, accum_mode,
                               pair_set, sum_rule, mem_cap)
    return _check(st, "ozaki_dgemm_ex") if check else st


def ozaki_dgemm_static(m, n, k, A, lda, B, ldb, C, ldc, slice_format, num_slices, k_block, accum_mode, check: bool = True) -> int:
    st = load().ozaki_dgemm_static(m, n, k, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, slice_format, num_slices, k_block, accum_mode)
    return _check(st, "ozaki_dgemm_static") if check else st


def ozaki_dgemm_scaled(m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, slice_format, num_slices, k_block, accum_mode,
                       check: bool = True) -> int:
    st = load().ozaki_dgemm_scaled(m, n, k, float(alpha), _ptr(A), lda, _ptr(B), ldb, float(beta), _ptr(C), ldc, slice_format,
                                   num_slices, k_block, accum_mode)
    return _check(st, "ozaki_dgemm_scaled") if check else st


def ozaki_count_slices(is_B, rows, k, X, ldx, slice_format, k_block) -> int:
    """Slices until the remainder of every vector is zero (MAX_SLICES + 1: more than the library can use)."""
    out = ctypes.c_int(0)
    _check(load().ozaki_count_slices(is_B, rows, k, _ptr(X), ldx, slice_format, k_block, ctypes.byref(out)), "ozaki_count_slices")
    return int(out.value)


def ozaki_split(is_B, rows, k, X, ldx, slice_format, num_slices, k_block, slices_out, exps_out, check: bool = True) -> int:
    st = load().ozaki_split(is_B, rows, k, _ptr(X), ldx, slice_format, num_slices, k_block, _ptr(slices_out), _ptr(exps_out))
    return _check(st, "ozaki_split") if check else st


def ozaki_pair_products(m, n, k, A, lda, B, ldb, slice_format, num_slices, k_block, P_out, pair_set=PAIRS_TRIANGLE, chained=0,
                        run_len_out=None, check: bool = True) -> int:
    st = load().ozaki_pair_products(m, n, k, _ptr(A), lda, _ptr(B), ldb, slice_format, num_slices, k_block, pair_set, chained,
                                    _ptr(P_out), _ptr(run_len_out))
    return _check(st, "ozaki_pair_products") if check else st


def ozaki_fp64_add_emulated(a, b, out, n) -> None:
    _check(load().ozaki_fp64_add_emulated(_ptr(a), _ptr(b), _ptr(out), n), "ozaki_fp64_add_emulated")
