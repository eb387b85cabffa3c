"""ctypes loader for libmixquant.so, the HIP (gfx950) library declared in include/mixquant.h.

There is no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MIXQUANT_LIB") or os.path.join(_HERE, "libmixquant.so")

MQ_OK = 0
MQ_OUT_BF16, MQ_OUT_FP32 = 0, 1
MQ_LAYOUT_LINEAR, MQ_LAYOUT_KTILE = 0, 1

_lib = None


class MixQuantError(RuntimeError):
    pass


def load() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MixQuantError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_20315_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.mq_codes_bytes.restype = ctypes.c_size_t
    lib.mq_codes_bytes.argtypes = [i64, i64]
    lib.mq_scales_bytes.restype = ctypes.c_size_t
    lib.mq_scales_bytes.argtypes = [i64, i64]
    lib.nvfp4_global_scale.restype = ci
    lib.nvfp4_global_scale.argtypes = [vp, i64, i64, i64, vp, vp]
    lib.nvfp4_quantize.restype = ci
    lib.nvfp4_quantize.argtypes = [vp, i64, i64, i64, vp, vp, vp, ci, vp]
    lib.nvfp4_quantize_silu_mul.restype = ci
    lib.nvfp4_quantize_silu_mul.argtypes = [vp, i64, i64, i64, vp, vp, vp, ci, vp, i64, vp]
    lib.nvfp4_quantize_rmsnorm.restype = ci
    lib.nvfp4_quantize_rmsnorm.argtypes = [vp, i64, i64, i64, vp, ctypes.c_float, vp, vp, vp, ci, vp, i64, vp]
    lib.nvfp4_relayout.restype = ci
    lib.nvfp4_relayout.argtypes = [vp, vp, vp, vp, i64, i64, ci, ci, vp]
    lib.nvfp4_gemm.restype = ci
    lib.nvfp4_gemm.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, i64, ci, ci, vp]
    lib.nvfp4_gemm_ws.restype = ci
    lib.nvfp4_gemm_ws.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, i64, ci, ci, vp, i64, vp]
    lib.nvfp4_gemm_noalloc.restype = ci
    lib.nvfp4_gemm_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, i64, ci, ci, vp]
    lib.mq_init.restype = ci
    lib.mq_init.argtypes = []
    lib.mq_gemm_workspace_bytes.restype = i64
    lib.mq_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    lib.bf16_gemm.restype = ci
    lib.bf16_gemm.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i64, ci, vp]
    lib.bf16_gemm_ws.restype = ci
    lib.bf16_gemm_ws.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i64, ci, vp, i64, vp]
    lib.mq_bf16_gemm_workspace_bytes.restype = i64
    lib.mq_bf16_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    lib.mq_mfma_probe.restype = ci
    lib.mq_mfma_probe.argtypes = [vp, ci, vp, ctypes.POINTER(ctypes.c_double)]
    lib.mq_status_string.restype = ctypes.c_char_p
    lib.mq_status_string.argtypes = [ci]
    lib.mq_last_hip_error.restype = ci
    lib.mq_last_hip_error.argtypes = []
    lib.mq_version.restype = ctypes.c_char_p
    lib.mq_version.argtypes = []
    _lib = lib
    return lib


def check(rc: int, what: str) -> None:
    if rc != MQ_OK:
        lib = load()
        msg = lib.mq_status_string(rc).decode()
        raise MixQuantError(f"{what}: {msg} (status {rc}, hipError {lib.mq_last_hip_error()})")
