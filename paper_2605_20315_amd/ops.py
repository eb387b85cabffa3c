"""Thin Python binding of the C ABI in include/mixquant.h: same names, argument marshalling only.

Every function takes torch tensors that live on the GPU, passes their device pointers and
the current HIP stream to the library, and returns the output tensors.  PyTorch provides
device memory and streams; all arithmetic runs in the HIP kernels.
"""
from __future__ import annotations

import torch

from . import _lib
from ._lib import (MQ_LAYOUT_KTILE, MQ_LAYOUT_LINEAR, MQ_OUT_BF16, MQ_OUT_FP32,  # noqa: F401
                   MixQuantError)

BLOCK = 16


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _need_gpu(*tensors) -> None:
    for t in tensors:
        if not t.is_cuda:
            raise MixQuantError("tensors must live on the GPU (the library has no CPU path)")


def _rows_k_ld(x: torch.Tensor):
    if x.dim() != 2 or x.stride(1) != 1:
        raise MixQuantError("expected a 2-D tensor whose last dimension is contiguous")
    ld = x.stride(0) if x.shape[0] > 1 else max(x.stride(0), x.shape[1])
    return x.shape[0], x.shape[1], ld


def nvfp4_global_scale(x_bf16: torch.Tensor, alpha_out: torch.Tensor | None = None) -> torch.Tensor:
    """alpha = max|x| / (6*448) as a one-element float32 device tensor."""
    _need_gpu(x_bf16)
    assert x_bf16.dtype == torch.bfloat16
    rows, K, ld = _rows_k_ld(x_bf16)
    alpha = alpha_out if alpha_out is not None else torch.empty(1, dtype=torch.float32, device=x_bf16.device)
    rc = _lib.load().nvfp4_global_scale(x_bf16.data_ptr(), rows, K, ld, alpha.data_ptr(), _stream())
    _lib.check(rc, "nvfp4_global_scale")
    return alpha


def nvfp4_quantize(x_bf16: torch.Tensor, alpha: torch.Tensor, codes: torch.Tensor | None = None,
                   scales: torch.Tensor | None = None, layout: int = MQ_LAYOUT_LINEAR):
    """Eq. 2 then Eq. 1 of Section 3.3.  Returns (codes uint8 [rows, K/2], scales uint8 [rows, K/16]);
    with MQ_LAYOUT_KTILE the same two buffers hold the bytes in K-step-major order."""
    _need_gpu(x_bf16, alpha)
    assert x_bf16.dtype == torch.bfloat16 and alpha.dtype == torch.float32
    rows, K, ld = _rows_k_ld(x_bf16)
    if K % BLOCK:
        _lib.check(2, "nvfp4_quantize")
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=x_bf16.device)
    if scales is None:
        scales = torch.empty((rows, K // BLOCK), dtype=torch.uint8, device=x_bf16.device)
    assert codes.is_contiguous() and scales.is_contiguous()
    rc = _lib.load().nvfp4_quantize(x_bf16.data_ptr(), rows, K, ld, alpha.data_ptr(),
                                    codes.data_ptr(), scales.data_ptr(), layout, _stream())
    _lib.check(rc, "nvfp4_quantize")
    return codes, scales


def _quant_outputs(rows: int, K: int, device, codes, scales, want_bf16: bool):
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=device)
    if scales is None:
        scales = torch.empty((rows, K // BLOCK), dtype=torch.uint8, device=device)
    assert codes.is_contiguous() and scales.is_contiguous()
    dbg = torch.empty((rows, K), dtype=torch.bfloat16, device=device) if want_bf16 else None
    return codes, scales, dbg


def nvfp4_quantize_silu_mul(gate_up_bf16: torch.Tensor, alpha: torch.Tensor, codes: torch.Tensor | None = None,
                            scales: torch.Tensor | None = None, layout: int = MQ_LAYOUT_LINEAR,
                            return_bf16: bool = False):
    """NVFP4 of silu(gate) * up for gate_up = [gate | up] of shape [rows, 2K] (fused producer).
    Returns (codes, scales), plus the BF16 tensor that was quantized when return_bf16 is set."""
    _need_gpu(gate_up_bf16, alpha)
    assert gate_up_bf16.dtype == torch.bfloat16 and alpha.dtype == torch.float32
    rows, k2, ld = _rows_k_ld(gate_up_bf16)
    if k2 % (2 * BLOCK):
        _lib.check(2, "nvfp4_quantize_silu_mul")
    K = k2 // 2
    codes, scales, p = _quant_outputs(rows, K, gate_up_bf16.device, codes, scales, return_bf16)
    rc = _lib.load().nvfp4_quantize_silu_mul(gate_up_bf16.data_ptr(), rows, K, ld, alpha.data_ptr(),
                                             codes.data_ptr(), scales.data_ptr(), layout,
                                             p.data_ptr() if p is not None else None, K, _stream())
    _lib.check(rc, "nvfp4_quantize_silu_mul")
    return (codes, scales, p) if return_bf16 else (codes, scales)


def nvfp4_quantize_rmsnorm(x_bf16: torch.Tensor, w_bf16: torch.Tensor, eps: float, alpha: torch.Tensor,
                           codes: torch.Tensor | None = None, scales: torch.Tensor | None = None,
                           layout: int = MQ_LAYOUT_LINEAR, return_bf16: bool = False):
    """NVFP4 of x / sqrt(mean(x^2) + eps) * w per row (fused producer).
    Returns (codes, scales), plus the BF16 tensor that was quantized when return_bf16 is set."""
    _need_gpu(x_bf16, w_bf16, alpha)
    assert x_bf16.dtype == torch.bfloat16 and w_bf16.dtype == torch.bfloat16 and alpha.dtype == torch.float32
    rows, K, ld = _rows_k_ld(x_bf16)
    assert w_bf16.shape == (K,) and w_bf16.is_contiguous()
    if K % 64:
        _lib.check(2, "nvfp4_quantize_rmsnorm")
    codes, scales, y = _quant_outputs(rows, K, x_bf16.device, codes, scales, return_bf16)
    rc = _lib.load().nvfp4_quantize_rmsnorm(x_bf16.data_ptr(), rows, K, ld, w_bf16.data_ptr(), float(eps),
                                            alpha.data_ptr(), codes.data_ptr(), scales.data_ptr(), layout,
                                            y.data_ptr() if y is not None else None, K, _stream())
    _lib.check(rc, "nvfp4_quantize_rmsnorm")
    return (codes, scales, y) if return_bf16 else (codes, scales)


def nvfp4_relayout(codes: torch.Tensor, scales: torch.Tensor, from_layout: int, to_layout: int):
    """Copy an NVFP4 tensor into the other byte order (offline weight pre-pack).  Returns (codes, scales)."""
    _need_gpu(codes, scales)
    rows, K = codes.shape[0], codes.shape[1] * 2
    assert codes.dtype == torch.uint8 and scales.dtype == torch.uint8
    assert codes.is_contiguous() and scales.is_contiguous() and scales.shape == (rows, K // BLOCK)
    oc, os_ = torch.empty_like(codes), torch.empty_like(scales)
    rc = _lib.load().nvfp4_relayout(codes.data_ptr(), scales.data_ptr(), oc.data_ptr(), os_.data_ptr(),
                                    rows, K, from_layout, to_layout, _stream())
    _lib.check(rc, "nvfp4_relayout")
    return oc, os_


def nvfp4_gemm(a_codes, a_scales, a_alpha, b_codes, b_scales, b_alpha, out: int = MQ_OUT_BF16,
               y: torch.Tensor | None = None, layout: int = MQ_LAYOUT_LINEAR) -> torch.Tensor:
    """Y[M, N] = dequant(A)[M, K] . dequant(B)[N, K]^T, FP32 accumulate, BF16 or FP32 out."""
    _need_gpu(a_codes, a_scales, a_alpha, b_codes, b_scales, b_alpha)
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    assert b_codes.shape[1] * 2 == K and a_scales.shape == (M, K // BLOCK) and b_scales.shape == (N, K // BLOCK)
    for t in (a_codes, a_scales, b_codes, b_scales):
        assert t.dtype == torch.uint8 and t.is_contiguous()
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16 if out == MQ_OUT_BF16 else torch.float32,
                        device=a_codes.device)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    rc = _lib.load().nvfp4_gemm(a_codes.data_ptr(), a_scales.data_ptr(), a_alpha.data_ptr(),
                                b_codes.data_ptr(), b_scales.data_ptr(), b_alpha.data_ptr(),
                                M, N, K, y.data_ptr(), ldy, out, layout, _stream())
    _lib.check(rc, "nvfp4_gemm")
    return y


def mq_init() -> None:
    """One-time set-up of the current device (kernel attributes, static scratch address); optional
    except before capturing the calls into a HIP graph."""
    _lib.check(_lib.load().mq_init(), "mq_init")


NOALLOC_SCRATCH_BYTES = 4 << 20


def nvfp4_gemm_noalloc(a_codes, a_scales, a_alpha, b_codes, b_scales, b_alpha, out: int = MQ_OUT_BF16,
                       y: torch.Tensor | None = None, layout: int = MQ_LAYOUT_LINEAR) -> torch.Tensor:
    """nvfp4_gemm_ws with the library's static scratch array as the workspace (allocates nothing;
    pass `y` to keep the binding from allocating the output)."""
    _need_gpu(a_codes, a_scales, a_alpha, b_codes, b_scales, b_alpha)
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    assert b_codes.shape[1] * 2 == K and a_scales.shape == (M, K // BLOCK) and b_scales.shape == (N, K // BLOCK)
    for t in (a_codes, a_scales, b_codes, b_scales):
        assert t.dtype == torch.uint8 and t.is_contiguous()
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16 if out == MQ_OUT_BF16 else torch.float32,
                        device=a_codes.device)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    rc = _lib.load().nvfp4_gemm_noalloc(a_codes.data_ptr(), a_scales.data_ptr(), a_alpha.data_ptr(),
                                        b_codes.data_ptr(), b_scales.data_ptr(), b_alpha.data_ptr(),
                                        M, N, K, y.data_ptr(), ldy, out, layout, _stream())
    _lib.check(rc, "nvfp4_gemm_noalloc")
    return y


def mq_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    """Workspace size that lets nvfp4_gemm_ws choose its K slabs freely (0: it would use none)."""
    return int(_lib.load().mq_gemm_workspace_bytes(M, N, K))


def nvfp4_gemm_ws(a_codes, a_scales, a_alpha, b_codes, b_scales, b_alpha, workspace: torch.Tensor | None,
                  out: int = MQ_OUT_BF16, y: torch.Tensor | None = None,
                  layout: int = MQ_LAYOUT_LINEAR) -> torch.Tensor:
    """nvfp4_gemm with a caller-owned workspace (any contiguous GPU tensor, or None) for the partial
    sums of small-M problems."""
    _need_gpu(a_codes, a_scales, a_alpha, b_codes, b_scales, b_alpha)
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    assert b_codes.shape[1] * 2 == K and a_scales.shape == (M, K // BLOCK) and b_scales.shape == (N, K // BLOCK)
    for t in (a_codes, a_scales, b_codes, b_scales):
        assert t.dtype == torch.uint8 and t.is_contiguous()
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16 if out == MQ_OUT_BF16 else torch.float32,
                        device=a_codes.device)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    ws_ptr, ws_bytes = 0, 0
    if workspace is not None:
        assert workspace.is_cuda and workspace.is_contiguous()
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    rc = _lib.load().nvfp4_gemm_ws(a_codes.data_ptr(), a_scales.data_ptr(), a_alpha.data_ptr(),
                                   b_codes.data_ptr(), b_scales.data_ptr(), b_alpha.data_ptr(),
                                   M, N, K, y.data_ptr(), ldy, out, layout, ws_ptr, ws_bytes, _stream())
    _lib.check(rc, "nvfp4_gemm_ws")
    return y


def bf16_gemm(x_bf16: torch.Tensor, w_bf16: torch.Tensor, out: int = MQ_OUT_BF16,
              y: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X . W^T with BF16 inputs and FP32 accumulation (the high-precision baseline)."""
    _need_gpu(x_bf16, w_bf16)
    assert x_bf16.dtype == torch.bfloat16 and w_bf16.dtype == torch.bfloat16
    M, K, ldx = _rows_k_ld(x_bf16)
    N, K2, ldw = _rows_k_ld(w_bf16)
    assert K == K2
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16 if out == MQ_OUT_BF16 else torch.float32,
                        device=x_bf16.device)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    rc = _lib.load().bf16_gemm(x_bf16.data_ptr(), ldx, w_bf16.data_ptr(), ldw, M, N, K,
                               y.data_ptr(), ldy, out, _stream())
    _lib.check(rc, "bf16_gemm")
    return y


def mq_bf16_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    """Workspace size that lets bf16_gemm_ws choose its K slabs freely (0: it would use none)."""
    return int(_lib.load().mq_bf16_gemm_workspace_bytes(M, N, K))


def bf16_gemm_ws(x_bf16: torch.Tensor, w_bf16: torch.Tensor, workspace: torch.Tensor | None,
                 out: int = MQ_OUT_BF16, y: torch.Tensor | None = None) -> torch.Tensor:
    """bf16_gemm with a caller-owned workspace (any contiguous GPU tensor, or None) for the partial
    sums of decode batches."""
    _need_gpu(x_bf16, w_bf16)
    assert x_bf16.dtype == torch.bfloat16 and w_bf16.dtype == torch.bfloat16
    M, K, ldx = _rows_k_ld(x_bf16)
    N, K2, ldw = _rows_k_ld(w_bf16)
    assert K == K2
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16 if out == MQ_OUT_BF16 else torch.float32,
                        device=x_bf16.device)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    ws_ptr, ws_bytes = 0, 0
    if workspace is not None:
        assert workspace.is_cuda and workspace.is_contiguous()
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    rc = _lib.load().bf16_gemm_ws(x_bf16.data_ptr(), ldx, w_bf16.data_ptr(), ldw, M, N, K,
                                  y.data_ptr(), ldy, out, ws_ptr, ws_bytes, _stream())
    _lib.check(rc, "bf16_gemm_ws")
    return y


def nvfp4_linear(x_bf16: torch.Tensor, alpha_x: torch.Tensor, w_codes, w_scales, alpha_w,
                 out: int = MQ_OUT_BF16, y: torch.Tensor | None = None, codes=None, scales=None,
                 layout: int = MQ_LAYOUT_LINEAR, workspace: torch.Tensor | None = None):
    """One prefill linear layer: quantize the activations, then the block-scaled GEMM (two library
    calls).  `layout` is the byte order of the weight arrays and of the activation arrays produced here."""
    xc, xs = nvfp4_quantize(x_bf16, alpha_x, codes, scales, layout)
    return nvfp4_gemm_ws(xc, xs, alpha_x, w_codes, w_scales, alpha_w, workspace, out, y, layout)


def mfma_probe(iters: int = 4000) -> float:
    """Enqueue the matrix-pipe rate probe on the current stream; returns the flop count of the launch."""
    import ctypes
    scratch = torch.zeros(1, dtype=torch.float32, device="cuda")
    flop = ctypes.c_double(0.0)
    rc = _lib.load().mq_mfma_probe(scratch.data_ptr(), iters, _stream(), ctypes.byref(flop))
    _lib.check(rc, "mq_mfma_probe")
    return flop.value
