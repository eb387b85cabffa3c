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


# Relative accuracy (in units of ||row|| * ||col||) that the FP32-output path is held to in every
# test: products are exact, only the FP32 accumulation rounds (measured worst: 9e-9).  The stated
# bound of the method is 1e-4; this tighter figure is what makes the strict BF16 rule below follow.
ACC_REL = 1e-7


def check_gemm_fp32(y: np.ndarray, y_ref: np.ndarray, norm_a: np.ndarray, norm_b: np.ndarray,
                    rel: float = 1e-4):
    """max |y - Y*| <= rel * ||row|| * ||col||, element by element.  Returns the worst ratio."""
    bound = np.outer(norm_a, norm_b)
    err = np.abs(y.astype(np.float64) - y_ref)
    ok = err <= rel * bound
    assert ok.all(), f"{(~ok).sum()} outputs beyond {rel}*||row||*||col||, worst err {err.max()}"
    worst = float((err / np.maximum(bound, 1e-300)).max())
    assert worst <= ACC_REL, f"FP32 accumulation error {worst:.2e} * ||row||*||col|| (exact products expected)"
    return worst


def check_gemm_bf16(y_bits: np.ndarray, y_ref: np.ndarray, norm_a: np.ndarray, norm_b: np.ndarray,
                    rel: float = 1e-4):
    """BF16 acceptance, two rules, both asserted.
    Band (every output): within 1 BF16 ulp of the correctly rounded value of some real number
    within rel*||row||*||col|| of Y* (an FP32-accumulated sum cannot do better where Y* is a
    near-cancellation).
    Strict (every output that is not a cancellation, |Y*| >= 2^8 * ACC_REL * ||row||*||col||, where an
    accumulation error of ACC_REL*||row||*||col|| is below one BF16 ulp of Y*): within 1 BF16 ulp of
    RNE(Y*) itself; and at least 99.99 % of all outputs when there are enough of them to say so.
    Returns the fraction of all outputs within 1 ulp of RNE(Y*)."""
    bound = np.outer(norm_a, norm_b)
    tau = rel * bound
    lo = bf16_ordinal(oracle.bf16_round(y_ref - tau)) - 1
    hi = bf16_ordinal(oracle.bf16_round(y_ref + tau)) + 1
    got = bf16_ordinal(y_bits)
    ok = (got >= lo) & (got <= hi)
    assert ok.all(), f"{(~ok).sum()} BF16 outputs outside the accepted interval"
    strict = np.abs(got - bf16_ordinal(oracle.bf16_round(y_ref))) <= 1
    plain = np.abs(y_ref) >= 256.0 * ACC_REL * bound
    bad = plain & ~strict
    assert not bad.any(), (f"{bad.sum()} non-cancellation BF16 outputs more than 1 ulp from RNE(Y*), e.g. at "
                           f"{np.argwhere(bad)[0].tolist()}")
    frac = float(strict.mean())
    if strict.size >= 10000:
        assert frac >= 0.9999, f"only {frac:.6f} of the BF16 outputs within 1 ulp of RNE(Y*)"
    return frac


def to_ktile(codes: np.ndarray, scales: np.ndarray):
    """The K-step-major byte order from the canonical one: the oracle's plain-loop permutation."""
    return oracle.to_ktile(codes, scales)
