"""GPU parity on seeded random shapes: quantize in either layout, multiply, compare with the
oracle.  Small enough that the oracle computes every output; shapes are drawn so that they hit
every workgroup shape of the register-direct NVFP4 kernel and the tiled BF16 kernels, the simple kernel (K % 64 != 0), ragged M and N,
and the decode-shape BF16 kernel."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import workloads as wl

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_bf16, host_bits, to_ktile

pytestmark = pytest.mark.gpu


def _cases():
    rng = np.random.default_rng(2026)
    out = []
    for _ in range(14):
        M = int(rng.integers(1, 700))
        N = int(rng.integers(1, 90)) * 8
        K = int(rng.integers(1, 40)) * 16
        out.append((M, N, K))
    out += [(4100, 4120, 64), (4352, 4352, 128), (3, 8, 16), (64, 8, 128), (65, 16, 128)]
    # large enough for the register-direct kernels (whole tiles and split K), every output checked
    for _ in range(6):
        M = int(rng.integers(1400, 3200))
        N = int(rng.integers(256, 520)) * 8
        K = int(rng.integers(1, 9)) * 64
        out.append((M, N, K))
    return out


@pytest.mark.parametrize("M,N,K", _cases())
def test_quantize_then_gemm_random_shape(M, N, K):
    rng = np.random.default_rng([M, N, K])
    x = wl.f32_to_bf16_bits((rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)))).astype(np.float32))
    w = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
    x[:, rng.integers(0, K)] = wl.f32_to_bf16_bits(np.float32(25.0) * wl.bf16_bits_to_f32(x[:, 0]))
    xd, wd = dev_bf16(x), dev_bf16(w)
    ax, aw = mq.nvfp4_global_scale(xd), mq.nvfp4_global_scale(wd)
    ax_ref, aw_ref = oracle.global_scale(x), oracle.global_scale(w)
    assert np.float32(ax.item()) == ax_ref and np.float32(aw.item()) == aw_ref
    xc_ref, xs_ref = oracle.quantize(x, ax_ref)
    wc_ref, ws_ref = oracle.quantize(w, aw_ref)
    layout = mq.MQ_LAYOUT_KTILE if K % 64 == 0 else mq.MQ_LAYOUT_LINEAR
    xc, xs = mq.nvfp4_quantize(xd, ax, layout=layout)
    wc, ws = mq.nvfp4_quantize(wd, aw, layout=layout)
    exp_x = to_ktile(xc_ref, xs_ref) if layout == mq.MQ_LAYOUT_KTILE else (xc_ref, xs_ref)
    exp_w = to_ktile(wc_ref, ws_ref) if layout == mq.MQ_LAYOUT_KTILE else (wc_ref, ws_ref)
    assert np.array_equal(xc.cpu().numpy(), exp_x[0]) and np.array_equal(xs.cpu().numpy(), exp_x[1])
    assert np.array_equal(wc.cpu().numpy(), exp_w[0]) and np.array_equal(ws.cpu().numpy(), exp_w[1])

    a = oracle.dequantize(xc_ref, xs_ref, ax_ref)
    b = oracle.dequantize(wc_ref, ws_ref, aw_ref)
    ref = oracle.gemm_f64(a, b)
    na, nb = oracle.row_norms(a), oracle.row_norms(b)
    y16 = mq.nvfp4_gemm(xc, xs, ax, wc, ws, aw, mq.MQ_OUT_BF16, layout=layout)
    y32 = mq.nvfp4_gemm(xc, xs, ax, wc, ws, aw, mq.MQ_OUT_FP32, layout=layout)
    torch.cuda.synchronize()
    check_gemm_bf16(host_bits(y16), ref, na, nb)
    check_gemm_fp32(y32.cpu().numpy(), ref, na, nb)

    if K % 8 == 0:
        a, b = oracle.bf16_to_f64(x), oracle.bf16_to_f64(w)
        ref = oracle.gemm_f64(a, b)
        yb = mq.bf16_gemm(xd, wd, mq.MQ_OUT_BF16)
        torch.cuda.synchronize()
        check_gemm_bf16(host_bits(yb), ref, oracle.row_norms(a), oracle.row_norms(b))
