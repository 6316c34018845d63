"""Binding of libkn_peaks.so: what this GPU reaches on a plain copy, a read-only sweep, and register-only MFMA /
FMA / sine loops.  The benchmark quotes its kernels against these next to the datasheet peaks."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkn_peaks.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (its HIP runtime must be the one in the process)
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libkn_peaks.so has not been built (run paper_2103_13744_amd/build.py)")
        L = C.CDLL(LIB_PATH)
        vp, i64, dp = C.c_void_p, C.c_int64, C.POINTER(C.c_double)
        L.kn_peak_copy.argtypes = [vp, vp, vp, i64, C.c_int, dp]
        L.kn_peak_read.argtypes = [vp, vp, i64, vp, C.c_int, dp]
        L.kn_peak_mfma.argtypes = [vp, C.c_int, vp, C.c_int, C.c_int, dp]
        L.kn_peak_valu.argtypes = [vp, C.c_int, vp, C.c_int, C.c_int, dp]
        _lib = L
    return _lib


def measure_peaks(copy_bytes: int = 1 << 30, reps: int = 5) -> dict:
    """-> {"hbm_copy_gbps", "hbm_read_gbps", "mfma_f16_tflops", "mfma_bf16_tflops", "mfma_f32_tflops",
    "valu_fma_f32_tflops", "valu_sin_tops"}, measured on the current device and stream."""
    import torch
    L = _load()
    st = torch.cuda.current_stream().cuda_stream
    src = torch.empty(copy_bytes // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    out = torch.empty(256 * 8 * 256, dtype=torch.float32, device="cuda")
    v = C.c_double()

    def call(fn, *args):
        rc = fn(*args, C.byref(v))
        if rc != 0:
            raise RuntimeError("peak micro-benchmark failed with status %d" % rc)
        return v.value

    res = {
        "hbm_copy_gbps": call(L.kn_peak_copy, st, src.data_ptr(), dst.data_ptr(), copy_bytes, reps) / 1e9,
        "hbm_read_gbps": call(L.kn_peak_read, st, src.data_ptr(), copy_bytes, out.data_ptr(), reps) / 1e9,
        "mfma_f16_tflops": call(L.kn_peak_mfma, st, 0, out.data_ptr(), 20000, reps) / 1e12,
        "mfma_bf16_tflops": call(L.kn_peak_mfma, st, 1, out.data_ptr(), 20000, reps) / 1e12,
        "mfma_f32_tflops": call(L.kn_peak_mfma, st, 2, out.data_ptr(), 10000, reps) / 1e12,
        "valu_fma_f32_tflops": call(L.kn_peak_valu, st, 0, out.data_ptr(), 20000, reps) / 1e12,
        "valu_sin_tops": call(L.kn_peak_valu, st, 1, out.data_ptr(), 10000, reps) / 1e12,
    }
    torch.cuda.synchronize()
    return res
