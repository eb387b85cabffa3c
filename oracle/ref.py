"""ctypes loader and numpy marshalling for the C oracle (``nvfp4_ref.c``).

TEST INFRASTRUCTURE ONLY: no arithmetic of the method is done in this file; every function
forwards to the C routine of the same name.  Arrays are host numpy arrays:
BF16 tensors are ``uint16`` bit patterns, codes/scales are ``uint8``, reals are ``float64``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

BLOCK = 16  # g, Section 3.3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nvfp4_ref.c")
_LIB = os.path.join(_HERE, "libnvfp4_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``nvfp4_ref.c`` with gcc (no-op when the library is newer than the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
             _SRC, "-lm", "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    i64, f32, f64, vp, u8, u16 = (ctypes.c_int64, ctypes.c_float, ctypes.c_double,
                                  ctypes.c_void_p, ctypes.c_uint8, ctypes.c_uint16)
    sig = {
        "nvfp4_ref_e2m1_value": (f64, [ctypes.c_int]),
        "nvfp4_ref_e4m3_value": (f64, [ctypes.c_int]),
        "nvfp4_ref_e4m3_round": (u8, [f32]),
        "nvfp4_ref_fp4_round": (u8, [f32]),
        "nvfp4_ref_bf16_round": (u16, [f64]),
        "nvfp4_ref_global_scale": (f32, [vp, i64, i64, i64]),
        "nvfp4_ref_quantize": (ctypes.c_int, [vp, i64, i64, i64, f32, vp, vp]),
        "nvfp4_ref_dequantize": (ctypes.c_int, [vp, vp, f32, i64, i64, vp]),
        "nvfp4_ref_relayout": (ctypes.c_int, [vp, vp, vp, vp, i64, i64, ctypes.c_int]),
        "nvfp4_ref_bf16_to_f64": (None, [vp, i64, i64, i64, vp]),
        "nvfp4_ref_gemm_f64": (None, [vp, vp, i64, i64, i64, vp]),
        "nvfp4_ref_silu_mul_f64": (None, [vp, i64, i64, i64, vp]),
        "nvfp4_ref_rmsnorm_f64": (None, [vp, i64, i64, i64, vp, f64, vp]),
        "nvfp4_ref_row_norms": (None, [vp, i64, i64, vp]),
        "nvfp4_ref_bf16_round_array": (None, [vp, i64, vp]),
        "nvfp4_ref_num_threads": (ctypes.c_int, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _rows_k_ld(x: np.ndarray):
    assert x.ndim == 2 and x.strides[1] == x.itemsize, "rows must be contiguous"
    return x.shape[0], x.shape[1], x.strides[0] // x.itemsize if x.shape[0] > 1 else x.shape[1]


def e2m1_value(code: int) -> float:
    return _load().nvfp4_ref_e2m1_value(int(code))


def e4m3_value(byte: int) -> float:
    return _load().nvfp4_ref_e4m3_value(int(byte))


def e4m3_round(s: float) -> int:
    """Pi_E4M3 of Eq. 2; ``s`` is taken as a binary32 value."""
    return int(_load().nvfp4_ref_e4m3_round(np.float32(s).item()))


def fp4_round(y: float) -> int:
    """Pi_FP4 of Eq. 1; ``y`` is taken as a binary32 value."""
    return int(_load().nvfp4_ref_fp4_round(np.float32(y).item()))


def bf16_round(v) -> np.ndarray:
    """binary64 -> BF16 bit patterns, nearest-even, one rounding."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().nvfp4_ref_bf16_round_array(_ptr(v), v.size, _ptr(out))
    return out


def global_scale(x_bf16: np.ndarray) -> np.float32:
    assert x_bf16.dtype == np.uint16
    rows, K, ld = _rows_k_ld(x_bf16)
    return np.float32(_load().nvfp4_ref_global_scale(_ptr(x_bf16), rows, K, ld))


def quantize(x_bf16: np.ndarray, alpha):
    """Eq. 2 then Eq. 1 on a [rows, K] BF16 tensor.  Returns (codes [rows,K/2], scales [rows,K/16])."""
    assert x_bf16.dtype == np.uint16
    rows, K, ld = _rows_k_ld(x_bf16)
    assert K % BLOCK == 0
    codes = np.empty((rows, K // 2), dtype=np.uint8)
    scales = np.empty((rows, K // BLOCK), dtype=np.uint8)
    rc = _load().nvfp4_ref_quantize(_ptr(x_bf16), rows, K, ld, np.float32(alpha).item(),
                                    _ptr(codes), _ptr(scales))
    assert rc == 0
    return codes, scales


def dequantize(codes: np.ndarray, scales: np.ndarray, alpha) -> np.ndarray:
    """x_hat = alpha * sigma * q in binary64 (exact)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    rows, K = codes.shape[0], codes.shape[1] * 2
    assert scales.shape == (rows, K // BLOCK)
    out = np.empty((rows, K), dtype=np.float64)
    rc = _load().nvfp4_ref_dequantize(_ptr(codes), _ptr(scales), np.float32(alpha).item(),
                                      rows, K, _ptr(out))
    assert rc == 0
    return out


def _relayout(codes: np.ndarray, scales: np.ndarray, to_ktile_flag: int):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    rows, K = codes.shape[0], codes.shape[1] * 2
    assert K % 64 == 0 and scales.shape == (rows, K // BLOCK)
    oc, os_ = np.empty_like(codes), np.empty_like(scales)
    rc = _load().nvfp4_ref_relayout(_ptr(codes), _ptr(scales), _ptr(oc), _ptr(os_), rows, K, to_ktile_flag)
    assert rc == 0
    return oc, os_


def to_ktile(codes: np.ndarray, scales: np.ndarray):
    """Canonical byte order -> K-step-major byte order (same array shapes, permuted bytes)."""
    return _relayout(codes, scales, 1)


def from_ktile(codes: np.ndarray, scales: np.ndarray):
    """K-step-major byte order -> canonical byte order."""
    return _relayout(codes, scales, 0)


def bf16_to_f64(x_bf16: np.ndarray) -> np.ndarray:
    assert x_bf16.dtype == np.uint16
    rows, K, ld = _rows_k_ld(x_bf16)
    out = np.empty((rows, K), dtype=np.float64)
    _load().nvfp4_ref_bf16_to_f64(_ptr(x_bf16), rows, K, ld, _ptr(out))
    return out


def silu_mul_f64(gate_up_bf16: np.ndarray) -> np.ndarray:
    """silu(gate) * up in binary64; gate = columns [0, K), up = columns [K, 2K) of a [rows, 2K] BF16 array."""
    assert gate_up_bf16.dtype == np.uint16 and gate_up_bf16.shape[1] % 2 == 0
    rows, k2, ld = _rows_k_ld(gate_up_bf16)
    out = np.empty((rows, k2 // 2), dtype=np.float64)
    _load().nvfp4_ref_silu_mul_f64(_ptr(gate_up_bf16), rows, k2 // 2, ld, _ptr(out))
    return out


def rmsnorm_f64(x_bf16: np.ndarray, w_bf16: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * w per row, in binary64; x [rows, K] and w [K] are BF16 bit patterns."""
    assert x_bf16.dtype == np.uint16 and w_bf16.dtype == np.uint16 and w_bf16.shape == (x_bf16.shape[1],)
    rows, K, ld = _rows_k_ld(x_bf16)
    w = np.ascontiguousarray(w_bf16)
    out = np.empty((rows, K), dtype=np.float64)
    _load().nvfp4_ref_rmsnorm_f64(_ptr(x_bf16), rows, K, ld, _ptr(w), float(eps), _ptr(out))
    return out


def gemm_f64(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """y[m,n] = sum_k a[m,k] * b[n,k], binary64, k ascending."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2
    y = np.empty((M, N), dtype=np.float64)
    _load().nvfp4_ref_gemm_f64(_ptr(a), _ptr(b), M, N, K, _ptr(y))
    return y


def row_norms(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty(a.shape[0], dtype=np.float64)
    _load().nvfp4_ref_row_norms(_ptr(a), a.shape[0], a.shape[1], _ptr(out))
    return out


def num_threads() -> int:
    return int(_load().nvfp4_ref_num_threads())
