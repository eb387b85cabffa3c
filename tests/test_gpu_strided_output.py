"""GPU: the output of a product may be a column slice of a wider buffer (row stride > N, e.g. one
projection written into a fused buffer).  Every kernel family must write exactly the [M, N] block:
the columns beyond N and the rows beyond M keep their sentinel, and the block equals, bit for
bit, what the same call writes into a dense buffer (the kernel choice does not depend on the
stride and every kernel sums in a fixed order).  The dense results themselves are checked
against the oracle in test_gpu_gemm.py and test_gpu_random_shapes.py; one case per family is
checked against it here as well."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_scalar, dev_u8, host_bits, to_ktile

pytestmark = pytest.mark.gpu

SENTINEL = -7.0  # exactly representable in BF16 and FP32


def _strided(M, N, dtype, left, right, extra_rows=2):
    """[M + extra_rows, left + N + right] buffer of sentinels and the [M, N] view inside it."""
    ld = left + N + right
    assert ld % 8 == 0 and left % 8 == 0
    buf = torch.full((M + extra_rows, ld), SENTINEL, dtype=dtype, device="cuda")
    return buf, buf[:M, left:left + N]


def _assert_only_block_written(buf, M, N, left):
    rest = buf.clone()
    rest[:M, left:left + N] = SENTINEL
    assert bool((rest == SENTINEL).all()), "a kernel wrote outside its [M, N] block"


# (M, N, K): register-direct whole-K / split-in-two / split-in-four workgroups, the 128x128 LDS
# pipeline, the simple kernel (K % 64 != 0)
FP4_SHAPES = [(4093, 4072, 128), (2000, 4000, 192), (1000, 4000, 192), (300, 520, 128), (70, 40, 80)]


@pytest.mark.parametrize("M,N,K", FP4_SHAPES)
@pytest.mark.parametrize("out", [mq.MQ_OUT_BF16, mq.MQ_OUT_FP32])
def test_nvfp4_gemm_into_a_column_slice(M, N, K, out):
    rng = np.random.default_rng([M, N, K, out])
    ac = rng.integers(0, 256, size=(M, K // 2)).astype(np.uint8)
    asc = rng.integers(0x28, 0x48, size=(M, K // 16)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    bsc = rng.integers(0x28, 0x48, size=(N, K // 16)).astype(np.uint8)
    aa, ba = np.float32(0.75), np.float32(1.5)
    layout = mq.MQ_LAYOUT_KTILE if K % 64 == 0 else mq.MQ_LAYOUT_LINEAR
    ops = (to_ktile(ac, asc) + to_ktile(bc, bsc)) if layout == mq.MQ_LAYOUT_KTILE else (ac, asc, bc, bsc)
    d = [dev_u8(t) for t in ops]
    a_al, b_al = dev_scalar(aa), dev_scalar(ba)
    dtype = torch.bfloat16 if out == mq.MQ_OUT_BF16 else torch.float32
    dense = mq.nvfp4_gemm(d[0], d[1], a_al, d[2], d[3], b_al, out, layout=layout)
    left, right = 64, (-N) % 8 + 24
    buf, view = _strided(M, N, dtype, left, right)
    mq.nvfp4_gemm(d[0], d[1], a_al, d[2], d[3], b_al, out, view, layout)
    torch.cuda.synchronize()
    assert torch.equal(view, dense)
    _assert_only_block_written(buf, M, N, left)

    a = oracle.dequantize(ac, asc, aa)
    b = oracle.dequantize(bc, bsc, ba)
    ref = oracle.gemm_f64(a, b)
    if out == mq.MQ_OUT_BF16:
        check_gemm_bf16(host_bits(view), ref, oracle.row_norms(a), oracle.row_norms(b))
    else:
        check_gemm_fp32(view.cpu().numpy(), ref, oracle.row_norms(a), oracle.row_norms(b))


# direct-to-LDS 256x256 and 256x128 tiles, register-staged 128x128 tiles, simple kernel, decode kernel
BF16_SHAPES = [(4093, 4072, 128), (2040, 4088, 128), (300, 520, 128), (70, 40, 72), (16, 1000, 256), (3, 264, 128)]


@pytest.mark.parametrize("M,N,K", BF16_SHAPES)
@pytest.mark.parametrize("out", [mq.MQ_OUT_BF16, mq.MQ_OUT_FP32])
def test_bf16_gemm_into_a_column_slice(M, N, K, out):
    torch.manual_seed(M * 131 + N * 7 + K + out)
    x = torch.randn(M, K, device="cuda").bfloat16()
    w = (torch.randn(N, K, device="cuda") * K ** -0.5).bfloat16()
    dtype = torch.bfloat16 if out == mq.MQ_OUT_BF16 else torch.float32
    dense = mq.bf16_gemm(x, w, out)
    left, right = 8, (-N) % 8 + 40
    buf, view = _strided(M, N, dtype, left, right)
    mq.bf16_gemm(x, w, out, view)
    torch.cuda.synchronize()
    assert torch.equal(view, dense)
    _assert_only_block_written(buf, M, N, left)

    a, b = oracle.bf16_to_f64(host_bits(x)), oracle.bf16_to_f64(host_bits(w))
    ref = oracle.gemm_f64(a, b)
    if out == mq.MQ_OUT_BF16:
        check_gemm_bf16(host_bits(view), ref, oracle.row_norms(a), oracle.row_norms(b))
    else:
        check_gemm_fp32(view.cpu().numpy(), ref, oracle.row_norms(a), oracle.row_norms(b))
