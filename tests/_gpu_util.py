"""Helpers shared by the GPU parity tests: host<->device marshalling and the acceptance rules.

Nothing here computes the method: expected values always come from ``oracle``.
"""
import numpy as np
import torch

import oracle


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 BF16 bit patterns (host) -> torch.bfloat16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev_u8(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_scalar(v) -> torch.Tensor:
    return torch.tensor([float(np.float32(v))], dtype=torch.float32, device="cuda")


def host_bits(t: torch.Tensor) -> np.ndarray:
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_ordinal(bits: np.ndarray) -> np.ndarray:
    """Map BF16 bit patterns to integers whose order is the numeric order (-0 and +0 coincide)."""
    b = bits.astype(np.int64)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def check_gemm_fp32(y: np.ndarray, y_ref: np.ndarray, norm_a: np.ndarray, norm_b: np.ndarray,
                    rel: float = 1e-4):
    """max |y - Y*| <= rel * ||row|| * ||col||, element by element.  Returns the worst ratio."""
    bound = np.outer(norm_a, norm_b)
    err = np.abs(y.astype(np.float64) - y_ref)
    ok = err <= rel * bound
    assert ok.all(), f"{(~ok).sum()} outputs beyond {rel}*||row||*||col||, worst err {err.max()}"
    return float((err / np.maximum(bound, 1e-300)).max())


def check_gemm_bf16(y_bits: np.ndarray, y_ref: np.ndarray, norm_a: np.ndarray, norm_b: np.ndarray,
                    rel: float = 1e-4):
    """BF16 acceptance: the output must lie within 1 BF16 ulp of the correctly rounded value of
    some real number within rel*||row||*||col|| of Y* (an FP32-accumulated sum cannot do better
    where Y* is a near-cancellation).  Returns the fraction that is within 1 ulp of RNE(Y*) itself."""
    tau = rel * np.outer(norm_a, norm_b)
    lo = bf16_ordinal(oracle.bf16_round(y_ref - tau)) - 1
    hi = bf16_ordinal(oracle.bf16_round(y_ref + tau)) + 1
    got = bf16_ordinal(y_bits)
    ok = (got >= lo) & (got <= hi)
    assert ok.all(), f"{(~ok).sum()} BF16 outputs outside the accepted interval"
    strict = np.abs(got - bf16_ordinal(oracle.bf16_round(y_ref))) <= 1
    return float(strict.mean())


def to_ktile(codes: np.ndarray, scales: np.ndarray):
    """The K-step-major byte order, from the canonical linear one, by the documented index map:
    codes_ktile[t, r, j] = codes_linear[r, t*32 + j], scales_ktile[t, r, j] = scales_linear[r, t*4 + j]."""
    R, half_k = codes.shape
    T = half_k // 32
    assert half_k % 32 == 0 and scales.shape == (R, T * 4)
    ck = np.ascontiguousarray(codes.reshape(R, T, 32).transpose(1, 0, 2)).reshape(R, half_k)
    sk = np.ascontiguousarray(scales.reshape(R, T, 4).transpose(1, 0, 2)).reshape(R, T * 4)
    return ck, sk
