"""CPU oracle for the NVFP4 prefill linear path (Section 3.3, Eq. 1-2 of the Mix-Quant paper).

TEST INFRASTRUCTURE ONLY.  Importable from ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg.  The HIP library and its Python binding never import this package and
this package never imports them.  The arithmetic lives in ``nvfp4_ref.c`` (plain scalar C);
this file only loads it with ctypes and marshals numpy arrays.
"""
from .ref import (  # noqa: F401
    BLOCK,
    bf16_round,
    bf16_to_f64,
    build,
    dequantize,
    e2m1_value,
    e4m3_round,
    e4m3_value,
    fp4_round,
    from_ktile,
    gemm_f64,
    global_scale,
    num_threads,
    quantize,
    rmsnorm_f64,
    row_norms,
    silu_mul_f64,
    to_ktile,
)
