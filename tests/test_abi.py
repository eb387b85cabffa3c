"""Host-side checks of the C-ABI library: it loads without a GPU, exports every function that
include/mixquant.h declares, and its argument validation runs before any launch.  CPU only."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_20315_amd import _lib, build
    if not os.path.exists(_lib.LIB_PATH):
        build.build_library()
    return _lib.load()


def _declared_functions():
    names = []
    for header in HEADERS:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b([a-z][a-z0-9_]*)\s*\([^;{]*\)\s*;", text)
    return names


def test_header_declares_the_three_calls_of_the_path():
    names = _declared_functions()
    for required in ("nvfp4_quantize", "nvfp4_gemm", "bf16_gemm", "nvfp4_global_scale"):
        assert required in names


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 9
    for n in names:
        assert hasattr(lib, n), n


def test_size_helpers_and_status_strings(lib):
    assert lib.mq_codes_bytes(8192, 4096) == 8192 * 2048
    assert lib.mq_scales_bytes(8192, 4096) == 8192 * 256
    assert lib.mq_codes_bytes(4, 24) == 0 and lib.mq_scales_bytes(-1, 16) == 0
    for code in range(7):
        assert lib.mq_status_string(code).decode().startswith("MQ_")
    assert lib.mq_version().decode().count(".") == 1


def test_validation_rejects_bad_arguments_before_any_launch(lib):
    # no GPU is touched: every call below fails (or is a no-op) in host-side validation
    assert lib.nvfp4_quantize(None, 4, 24, 24, None, None, None, 0, None) == 2      # K % 16
    assert lib.nvfp4_quantize(None, 4, 64, 64, None, None, None, 0, None) == 1      # NULL
    assert lib.nvfp4_quantize(None, 0, 64, 64, None, None, None, 0, None) == 0      # empty: no-op
    assert lib.nvfp4_quantize(None, -1, 64, 64, None, None, None, 0, None) == 2
    assert lib.nvfp4_quantize(None, 4, 48, 48, None, None, None, 1, None) == 2      # KTILE needs K % 64
    assert lib.nvfp4_quantize(None, 4, 64, 64, None, None, None, 2, None) == 4      # unknown layout
    # producer-fused quantizers
    f = ctypes.c_float
    assert lib.nvfp4_quantize_silu_mul(None, 4, 24, 48, None, None, None, 0, None, 0, None) == 2   # K % 16
    assert lib.nvfp4_quantize_silu_mul(None, 4, 64, 100, None, None, None, 0, None, 0, None) == 2  # ld < 2K
    assert lib.nvfp4_quantize_silu_mul(None, 4, 64, 128, None, None, None, 0, None, 0, None) == 1  # NULL
    assert lib.nvfp4_quantize_silu_mul(None, 0, 64, 128, None, None, None, 1, None, 0, None) == 0  # empty
    assert lib.nvfp4_quantize_silu_mul(None, 4, 64, 128, None, None, None, 7, None, 0, None) == 4
    assert lib.nvfp4_quantize_rmsnorm(None, 4, 48, 48, None, f(1e-6), None, None, None, 0, None, 0, None) == 2
    assert lib.nvfp4_quantize_rmsnorm(None, 0, 64, 64, None, f(-1.0), None, None, None, 0, None, 0, None) == 4
    assert lib.nvfp4_quantize_rmsnorm(None, 0, 64, 64, None, f(1e-6), None, None, None, 0, None, 0, None) == 0
    assert lib.nvfp4_quantize_rmsnorm(None, 4, 64, 64, None, f(1e-6), None, None, None, 0, None, 0, None) == 1
    assert lib.nvfp4_gemm(None, None, None, None, None, None, 4, 4, 40, None, 8, 0, 0, None) == 2
    assert lib.nvfp4_gemm(None, None, None, None, None, None, 4, 4, 64, None, 8, 3, 0, None) == 4
    assert lib.nvfp4_gemm(None, None, None, None, None, None, 4, 4, 64, None, 8, 0, 5, None) == 4
    assert lib.nvfp4_gemm(None, None, None, None, None, None, 4, 4, 48, None, 8, 0, 1, None) == 2
    assert lib.nvfp4_gemm(None, None, None, None, None, None, 4, 4, 64, None, 8, 0, 0, None) == 1
    assert lib.nvfp4_gemm(None, None, None, None, None, None, 0, 4, 64, None, 8, 0, 0, None) == 0
    # the workspace variant validates like nvfp4_gemm, plus its two extra arguments
    assert lib.nvfp4_gemm_ws(None, None, None, None, None, None, 4, 4, 40, None, 8, 0, 0, None, 0, None) == 2
    assert lib.nvfp4_gemm_ws(None, None, None, None, None, None, 4, 4, 64, None, 8, 0, 0, None, -8, None) == 2
    assert lib.nvfp4_gemm_ws(None, None, None, None, None, None, 4, 4, 64, None, 8, 0, 0, None, 64, None) == 1
    assert lib.nvfp4_gemm_ws(None, None, None, None, None, None, 0, 4, 64, None, 8, 0, 0, None, 64, None) == 0
    # the allocation-free variant: same validation, no GPU touched on an argument error
    assert lib.nvfp4_gemm_noalloc(None, None, None, None, None, None, 4, 4, 40, None, 8, 0, 0, None) == 2
    assert lib.nvfp4_gemm_noalloc(None, None, None, None, None, None, 0, 4, 64, None, 8, 0, 0, None) == 0
    assert lib.bf16_gemm(None, 64, None, 64, 4, 4, 64, None, 8, 0, None) == 1
    assert lib.bf16_gemm(None, 32, None, 64, 4, 4, 64, None, 8, 0, None) == 2
    assert lib.nvfp4_global_scale(None, 4, 64, 64, None, None) == 1
    assert lib.bf16_gemm_ws(None, 64, None, 64, 4, 4, 64, None, 8, 0, None, 0, None) == 1
    assert lib.bf16_gemm_ws(None, 64, None, 64, 4, 4, 64, None, 8, 0, None, -1, None) == 2
    assert lib.bf16_gemm_ws(None, 64, None, 64, 0, 4, 64, None, 8, 0, None, 0, None) == 0


def test_workspace_size_query(lib):
    """Host-only: slabs of K across workgroups are offered only where they pay: at most 128 output
    tiles of 64x64 and a K long enough that the K steps taken off each wave outweigh the second
    pass; the size is slabs * M * N * 4 bytes and never exceeds one 64x64 FP32 tile per compute
    unit of the largest gfx950 part (256 x 16 KiB = 4 MiB)."""
    q = lib.mq_gemm_workspace_bytes
    assert q(8192, 4096, 4096) == 0          # 8192 tiles
    assert q(128, 28672, 4096) == 0          # 896 tiles of 64x64
    assert q(128, 4096, 4096) == 0           # 64 K steps: the one-launch small-tile kernel
    assert q(256, 4096, 14336) == 0          # 256 tiles of 64x64: every compute unit has one
    assert q(128, 4098, 14336) == 0          # N % 4 != 0
    assert q(128, 4096, 14320) == 0          # K % 64 != 0
    assert q(0, 4096, 4096) == 0 and q(128, 0, 4096) == 0 and q(128, 4096, 0) == 0
    for M, N, K in [(128, 4096, 14336), (64, 4096, 14336), (300, 1024, 8192), (17, 136, 65536)]:
        b = q(M, N, K)
        assert b > 0 and b % (M * N * 4) == 0
        slabs = b // (M * N * 4)
        tiles = -(-M // 64) * -(-N // 64)
        assert 2 <= slabs <= min(256 // tiles, K // 2048)      # at least four K steps for each of eight waves
        assert b <= 256 * 64 * 64 * 4


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2605_20315_amd as mq
    with pytest.raises(mq.MixQuantError):
        mq.bf16_gemm(torch.zeros(4, 8, dtype=torch.bfloat16), torch.zeros(4, 8, dtype=torch.bfloat16))
