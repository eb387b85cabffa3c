"""GPU parity of the producer-fused quantizers (Section 3.3: the quantizer fused with its
neighbours) against the CPU oracle.

The producer is floating point and decides integers (the codes), so the check has two parts:
 1. the BF16 tensor the kernel quantized (its optional output) is within 1 BF16 ulp of the
    oracle's binary64 producer rounded to BF16, and equal to it for almost every element;
 2. codes and scale bytes are bit-identical to the oracle quantizer applied to that same BF16
    tensor, in both layouts, and identical whether or not the BF16 tensor is written out.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import workloads as wl

from _gpu_util import bf16_ordinal, dev_bf16, dev_scalar, host_bits, to_ktile

pytestmark = pytest.mark.gpu


def _check_producer(p_gpu_bits, ref_f64, min_equal):
    ref_bits = oracle.bf16_round(ref_f64)
    d = np.abs(bf16_ordinal(p_gpu_bits).astype(np.int64) - bf16_ordinal(ref_bits).astype(np.int64))
    assert d.max() <= 1, f"producer off by {d.max()} BF16 ulps"
    equal = float((d == 0).mean())
    # a fraction only means something on enough elements: small tensors may miss by one element
    assert equal >= min_equal or int((d != 0).sum()) <= 1, equal
    return equal


def _check_quantized(run, p_bits, alpha):
    """run(layout, return_bf16) -> tensors; p_bits: the BF16 tensor the kernel says it quantized."""
    c_ref, s_ref = oracle.quantize(p_bits, alpha)
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        c, s, p = run(layout, True)
        c2, s2 = run(layout, False)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(p), p_bits)                # same producer values in every mode
        assert torch.equal(c, c2) and torch.equal(s, s2)
        ce, se = (c_ref, s_ref) if layout == mq.MQ_LAYOUT_LINEAR else to_ktile(c_ref, s_ref)
        assert np.array_equal(s.cpu().numpy(), se)
        assert np.array_equal(c.cpu().numpy(), ce)


@pytest.mark.parametrize("rows,K", [(1, 64), (37, 192), (256, 1024), (1000, 14336), (2051, 4096)])
def test_silu_mul_quantize(rows, K):
    rng = np.random.default_rng([rows, K, 1])
    gu = wl.f32_to_bf16_bits(np.concatenate([rng.standard_normal((rows, K)) * 2.0,
                                             rng.standard_normal((rows, K))], axis=1).astype(np.float32))
    gu[0, :16] = wl.f32_to_bf16_bits(np.array([-60, -30, -10, -1, -0.0, 0.0, 1e-20, 1, 10, 30, 60, 87, -87, 5, -5, 0.5],
                                              dtype=np.float32))      # extreme and tiny gates (exp(-g) stays finite in binary32)
    if rows > 2:
        gu[2, :K] = 0                                                  # a zero row (all-zero blocks)
    ref = oracle.silu_mul_f64(gu)
    alpha = oracle.global_scale(oracle.bf16_round(ref))
    gud, ad = dev_bf16(gu), dev_scalar(alpha)
    run = lambda layout, dbg: mq.nvfp4_quantize_silu_mul(gud, ad, layout=layout, return_bf16=dbg)
    _, _, p = run(mq.MQ_LAYOUT_LINEAR, True)
    torch.cuda.synchronize()
    p_bits = host_bits(p)
    equal = _check_producer(p_bits, ref, 0.999)
    _check_quantized(run, p_bits, alpha)
    print(f"\n[silu_mul rows={rows} K={K}] producer equal to RNE(binary64) on {equal:.6f} of the elements")


def test_silu_mul_row_stride_and_ktile_requirements():
    rng = np.random.default_rng(5)
    rows, K = 40, 128
    wide = torch.zeros((rows, 2 * K + 64), dtype=torch.bfloat16, device="cuda")
    gu = wl.f32_to_bf16_bits(rng.standard_normal((rows, 2 * K)).astype(np.float32))
    wide[:, :2 * K] = dev_bf16(gu)
    ref = oracle.bf16_round(oracle.silu_mul_f64(gu))
    alpha = oracle.global_scale(ref)
    c, s, p = mq.nvfp4_quantize_silu_mul(wide[:, :2 * K], dev_scalar(alpha), return_bf16=True)
    c_ref, s_ref = oracle.quantize(host_bits(p), alpha)
    assert np.array_equal(c.cpu().numpy(), c_ref) and np.array_equal(s.cpu().numpy(), s_ref)
    with pytest.raises(mq.MixQuantError):                          # K = 48: K-step-major needs K % 64 == 0
        mq.nvfp4_quantize_silu_mul(torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda"), dev_scalar(1.0),
                                   layout=mq.MQ_LAYOUT_KTILE)


@pytest.mark.parametrize("rows,K,eps", [(1, 64, 1e-6), (37, 192, 1e-5), (300, 4096, 1e-6), (77, 5120, 1e-6),
                                        (50, 8192, 1e-5), (1030, 1024, 0.0)])
def test_rmsnorm_quantize(rows, K, eps):
    rng = np.random.default_rng([rows, K, 2])
    x = wl.f32_to_bf16_bits((rng.standard_normal((rows, K)) * np.exp(rng.standard_normal((rows, 1)))).astype(np.float32))
    x[:, rng.integers(0, K)] = wl.f32_to_bf16_bits(np.float32(20.0) * wl.bf16_bits_to_f32(x[:, 0]))   # outlier channel
    if rows > 3 and eps > 0:
        x[3] = 0                                                       # zero row: y = 0, all-zero blocks
    w = wl.f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(K)).astype(np.float32))
    ref = oracle.rmsnorm_f64(x, w, eps)
    alpha = oracle.global_scale(oracle.bf16_round(ref))
    xd, wd, ad = dev_bf16(x), dev_bf16(w), dev_scalar(alpha)
    run = lambda layout, dbg: mq.nvfp4_quantize_rmsnorm(xd, wd, eps, ad, layout=layout, return_bf16=dbg)
    _, _, y = run(mq.MQ_LAYOUT_LINEAR, True)
    torch.cuda.synchronize()
    y_bits = host_bits(y)
    equal = _check_producer(y_bits, ref, 0.9999)
    _check_quantized(run, y_bits, alpha)
    print(f"\n[rmsnorm rows={rows} K={K}] producer equal to RNE(binary64) on {equal:.6f} of the elements")


def test_fused_quantizers_feed_the_gemm():
    """End to end: rmsnorm -> quantize -> GEMM equals quantize(BF16 producer output) -> GEMM bit for bit."""
    rng = np.random.default_rng(9)
    M, K, N = 300, 1024, 264
    x = dev_bf16(wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)))
    g = dev_bf16(wl.f32_to_bf16_bits(np.ones(K, dtype=np.float32)))
    w = dev_bf16(wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32)))
    aw = mq.nvfp4_global_scale(w)
    wc, ws = mq.nvfp4_quantize(w, aw, layout=mq.MQ_LAYOUT_KTILE)
    ax = dev_scalar(6.0 / 2688.0)
    c1, s1, y = mq.nvfp4_quantize_rmsnorm(x, g, 1e-6, ax, layout=mq.MQ_LAYOUT_KTILE, return_bf16=True)
    c2, s2 = mq.nvfp4_quantize(y, ax, layout=mq.MQ_LAYOUT_KTILE)
    assert torch.equal(c1, c2) and torch.equal(s1, s2)
    out1 = mq.nvfp4_gemm(c1, s1, ax, wc, ws, aw, mq.MQ_OUT_BF16, layout=mq.MQ_LAYOUT_KTILE)
    out2 = mq.nvfp4_gemm(c2, s2, ax, wc, ws, aw, mq.MQ_OUT_BF16, layout=mq.MQ_LAYOUT_KTILE)
    assert torch.equal(out1, out2)
