"""GPU parity of the one-launch small-tile NVFP4 kernel (64x64 output tiles, K split over the
waves of a workgroup and summed through LDS in wave order), the path of prefill chunks of up to a
few hundred tokens.  Every output is compared with the oracle's FP64 product of the dequantized
operands; shapes cover eight, four and fewer waves per tile (K of 2 .. 224 steps, including
counts that the waves do not divide), a single wave (no reduction), ragged M and N, N that is
not a multiple of 32, one row, strided outputs with guard bands, both byte orders and both
output types, and every K position of a K step on its own."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_scalar, dev_u8, host_bits, to_ktile

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed, lo=0x28, hi=0x48):
    rng = np.random.default_rng([M, N, K, seed])
    ac = rng.integers(0, 256, size=(M, K // 2)).astype(np.uint8)
    asc = rng.integers(lo, hi, size=(M, K // 16)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    bsc = rng.integers(lo, hi, size=(N, K // 16)).astype(np.uint8)
    return ac, asc, np.float32(0.75), bc, bsc, np.float32(1.5)


# tiles of 64x64 <= 512 selects the kernel; waves per tile = 8 up to 256 tiles, else 4, capped at
# (K / 64) / 2.  (64, 4096, 4096): 64 tiles x 8 waves x 8 steps; (128, 6144, 4096): 192 x 8;
# (256, 6144, 1024): 384 tiles x 4 waves; (250, 1000, 704): 11 K steps over 5 waves (3, 3, 3, 2, 0);
# (77, 200, 448): 7 steps over 3 waves; (33, 72, 128): one wave; (1, 8, 64): one K step;
# (64, 4096, 14336): without a workspace, 224 steps over 8 waves; (500, 4000, 192): 504 tiles.
SHAPES = [(64, 4096, 4096), (128, 6144, 4096), (256, 6144, 1024), (250, 1000, 704), (77, 200, 448),
          (33, 72, 128), (1, 8, 64), (64, 4096, 14336), (500, 4000, 192), (129, 130, 1280)]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("layout", [mq.MQ_LAYOUT_KTILE, mq.MQ_LAYOUT_LINEAR])
def test_small_tile_kernel_against_oracle(M, N, K, layout):
    print(f"\n[case] small tiles M={M} N={N} K={K} layout={layout}", flush=True)
    ac, asc, aa, bc, bsc, ba = _operands(M, N, K, 0)
    a, b = oracle.dequantize(ac, asc, aa), oracle.dequantize(bc, bsc, ba)
    ref, na, nb = oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b)
    arrs = (to_ktile(ac, asc) + to_ktile(bc, bsc)) if layout == mq.MQ_LAYOUT_KTILE else (ac, asc, bc, bsc)
    d = [dev_u8(t) for t in arrs]
    a_al, b_al = dev_scalar(aa), dev_scalar(ba)
    ld = (N + 7) // 8 * 8 + 8
    b32 = torch.full((M + 1, ld), -7.0, dtype=torch.float32, device="cuda")
    b16 = torch.full((M + 1, ld), -7.0, dtype=torch.bfloat16, device="cuda")
    y32 = mq.nvfp4_gemm(d[0], d[1], a_al, d[2], d[3], b_al, mq.MQ_OUT_FP32, b32[:M, :N], layout)
    y16 = mq.nvfp4_gemm(d[0], d[1], a_al, d[2], d[3], b_al, mq.MQ_OUT_BF16, b16[:M, :N], layout)
    b16b = torch.empty((M, ld), dtype=torch.bfloat16, device="cuda")
    again = mq.nvfp4_gemm(d[0], d[1], a_al, d[2], d[3], b_al, mq.MQ_OUT_BF16, b16b[:, :N], layout)
    torch.cuda.synchronize()
    check_gemm_fp32(y32.cpu().numpy(), ref, na, nb)
    check_gemm_bf16(host_bits(y16), ref, na, nb)
    assert torch.equal(y32.to(torch.bfloat16), y16)       # BF16 = nearest-even rounding of the FP32 sums
    assert torch.equal(again, y16)                        # bit-identical from run to run
    for buf in (b32, b16):                                # nothing written outside [M, N]
        assert bool((buf[M:] == -7.0).all()) and bool((buf[:, N:] == -7.0).all())


def test_small_tile_kernel_extreme_scales():
    M, N, K = 70, 96, 1024
    ac, asc, aa, bc, bsc, ba = _operands(M, N, K, 1, 0x00, 0x7F)   # every E4M3 byte incl. subnormals and 448
    a, b = oracle.dequantize(ac, asc, 1.0), oracle.dequantize(bc, bsc, 1.0)
    y = mq.nvfp4_gemm(dev_u8(ac), dev_u8(asc), dev_scalar(1.0), dev_u8(bc), dev_u8(bsc), dev_scalar(1.0),
                      mq.MQ_OUT_FP32)
    torch.cuda.synchronize()
    check_gemm_fp32(y.cpu().numpy(), oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b))


@pytest.mark.parametrize("K", [128, 1024])
def test_small_tile_kernel_k_positions_one_hot(K):
    """Row r of A holds a single 1.0 at k = r % K, so Y[r, n] = B_hat[n, r % K] exactly: every K
    position of every wave's K range must meet its partner and nothing else."""
    M, N = 2 * K if K == 128 else K, 200
    ac = np.zeros((M, K // 2), dtype=np.uint8)
    asc = np.full((M, K // 16), 0x38, dtype=np.uint8)
    k = np.arange(M) % K
    ac[np.arange(M), k // 2] = (0x2 << (4 * (k & 1))).astype(np.uint8)
    rng = np.random.default_rng(K)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    bsc = rng.integers(0x28, 0x48, size=(N, K // 16)).astype(np.uint8)
    b = oracle.dequantize(bc, bsc, 1.0)
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        arrs = (to_ktile(ac, asc) + to_ktile(bc, bsc)) if layout == mq.MQ_LAYOUT_KTILE else (ac, asc, bc, bsc)
        d = [dev_u8(t) for t in arrs]
        y = mq.nvfp4_gemm(d[0], d[1], dev_scalar(1.0), d[2], d[3], dev_scalar(1.0), mq.MQ_OUT_FP32, layout=layout)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().astype(np.float64), b.T[k])
