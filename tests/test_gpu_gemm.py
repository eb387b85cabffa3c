"""GPU parity: nvfp4_gemm and bf16_gemm (C ABI, HIP kernels) against the CPU oracle's FP64
product of the dequantized operands (Section 3.3).

Acceptance: FP32 output |y - Y*| <= 1e-4 * ||row|| * ||col||; BF16 output within 1 BF16 ulp of
the correct rounding of a value inside that same band around Y* (see _gpu_util.check_gemm_bf16).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import workloads as wl

from _gpu_util import (check_gemm_bf16, check_gemm_fp32, dev_bf16, dev_scalar, dev_u8, host_bits, to_ktile)

pytestmark = pytest.mark.gpu


def _rand_nvfp4(rng, rows, K, lo=0x28, hi=0x48):
    scales = rng.integers(lo, hi, size=(rows, K // 16)).astype(np.uint8)
    codes = rng.integers(0, 256, size=(rows, K // 2)).astype(np.uint8)
    return codes, scales


def _gpu_gemm(ac, asc, aa, bc, bsc, ba, out, layout=None):
    """Operands are given in the canonical linear order; layout=None alternates: the K-step-major
    layout for the BF16 output and the linear one for FP32, so both are exercised on every case."""
    M, N = ac.shape[0], bc.shape[0]
    if layout is None:
        layout = mq.MQ_LAYOUT_KTILE if (out == mq.MQ_OUT_BF16 and ac.shape[1] % 32 == 0) else mq.MQ_LAYOUT_LINEAR
    if layout == mq.MQ_LAYOUT_KTILE:
        ac, asc = to_ktile(ac, asc)
        bc, bsc = to_ktile(bc, bsc)
    ld = (N + 7) // 8 * 8                     # the row stride must be a multiple of 8 elements
    buf = torch.empty((M, ld), dtype=torch.bfloat16 if out == mq.MQ_OUT_BF16 else torch.float32, device="cuda")
    y = mq.nvfp4_gemm(dev_u8(ac), dev_u8(asc), dev_scalar(aa), dev_u8(bc), dev_u8(bsc), dev_scalar(ba), out,
                      buf[:, :N], layout)
    torch.cuda.synchronize()
    return y


def _check_both(ac, asc, aa, bc, bsc, ba):
    a = oracle.dequantize(ac, asc, aa)
    b = oracle.dequantize(bc, bsc, ba)
    ref = oracle.gemm_f64(a, b)
    na, nb = oracle.row_norms(a), oracle.row_norms(b)
    y32 = _gpu_gemm(ac, asc, aa, bc, bsc, ba, mq.MQ_OUT_FP32).cpu().numpy()
    worst = check_gemm_fp32(y32, ref, na, nb)
    y16 = host_bits(_gpu_gemm(ac, asc, aa, bc, bsc, ba, mq.MQ_OUT_BF16))
    strict = check_gemm_bf16(y16, ref, na, nb)
    return worst, strict


def test_tiny_config_full_output():
    cfg = wl.configs()[0]
    x, w = wl.activation(cfg, 0), wl.weight(cfg, 0)
    ax, aw = oracle.global_scale(x), oracle.global_scale(w)
    xc, xs = oracle.quantize(x, ax)
    wc, ws = oracle.quantize(w, aw)
    worst, strict = _check_both(xc, xs, ax, wc, ws, aw)
    assert worst < 1e-5          # exact products, FP32 accumulation only
    assert strict > 0.999


def test_tiny_config_end_to_end_through_the_gpu_quantizer():
    cfg = wl.configs()[0]
    x, w = wl.activation(cfg, 0), wl.weight(cfg, 0)
    xd, wd = dev_bf16(x), dev_bf16(w)
    ax, aw = mq.nvfp4_global_scale(xd), mq.nvfp4_global_scale(wd)
    wc, ws = mq.nvfp4_quantize(wd, aw, layout=mq.MQ_LAYOUT_KTILE)
    y = mq.nvfp4_linear(xd, ax, wc, ws, aw, layout=mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    axr, awr = oracle.global_scale(x), oracle.global_scale(w)
    a = oracle.dequantize(*oracle.quantize(x, axr), axr)
    b = oracle.dequantize(*oracle.quantize(w, awr), awr)
    check_gemm_bf16(host_bits(y), oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b))


@pytest.mark.parametrize("M,N,K", [
    (1, 16, 64), (5, 48, 128), (31, 16, 64), (33, 80, 192), (127, 144, 256), (129, 272, 64),
    (257, 130, 320), (300, 1000, 512), (513, 257, 1024), (64, 64, 4096),
    (7, 16, 16), (19, 33, 48), (40, 24, 144),          # K not a multiple of 64: simple kernel
])
def test_ragged_shapes(M, N, K):
    rng = np.random.default_rng(M * 131 + N * 17 + K)
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    _check_both(ac, asc, 0.013, bc, bsc, 0.0021)


@pytest.mark.parametrize("K", [128, 192, 320])
def test_large_tile_path_with_ragged_edges(K):
    """16 x 32 tiles of 256x256 select the register-direct kernel with whole tiles (persistent
    workgroups, two tiles each), with M and N off the tile grid; an odd number of K steps makes
    its K loop run one step past the end with zeroed scales.  Both layouts, both output types."""
    rng = np.random.default_rng(5 + K)
    M, N = 256 * 15 + 77, 256 * 31 + 40
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    a = oracle.dequantize(ac, asc, 0.5)
    b = oracle.dequantize(bc, bsc, 0.25)
    rows = np.unique(np.concatenate([np.arange(0, M, 251), np.arange(M - 80, M), [127, 128, 255, 256, 257]]))
    ref = oracle.gemm_f64(a[rows], b)
    na, nb = oracle.row_norms(a[rows]), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        y32 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_FP32, layout)
        check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
        y16 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_BF16, layout)
        check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
        # the two output types come from the same accumulators
        assert torch.equal(y32.to(torch.bfloat16), y16)


@pytest.mark.parametrize("M,N", [(256 * 16, 256 * 32), (2048, 4096), (1024, 4096)])
def test_register_direct_k_positions_one_hot(M, N):
    """Register-direct kernel, whole tiles and K split two and four ways: an element at every k of a K step must
    meet exactly its partner.  A is a tall stack of one-hot rows (row r has a 1.0 at k = r % K),
    so Y[r, n] = B_hat[n, r % K]."""
    K = 128
    ac = np.zeros((M, K // 2), dtype=np.uint8)
    asc = np.full((M, K // 16), 0x38, dtype=np.uint8)
    k = np.arange(M) % K
    ac[np.arange(M), k // 2] = (0x2 << (4 * (k & 1))).astype(np.uint8)
    rng = np.random.default_rng(18)
    bc, bsc = _rand_nvfp4(rng, N, K)
    b = oracle.dequantize(bc, bsc, 1.0)
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        y = _gpu_gemm(ac, asc, 1.0, bc, bsc, 1.0, mq.MQ_OUT_FP32, layout).cpu().numpy().astype(np.float64)
        assert np.array_equal(y, b.T[k])


@pytest.mark.parametrize("K", [64, 192, 448])
def test_split_k_path_with_ragged_edges(K):
    """256 workgroup tiles of 256x128 select the register-direct kernel with K split over wave
    pairs (one K step: the second half is empty; three and seven: halves of unequal length, the
    second ending on a zeroed extra step).  The BF16 baseline takes its 256x128 configuration."""
    rng = np.random.default_rng(15 + K)
    M, N = 2000, 4000
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    a = oracle.dequantize(ac, asc, 0.5)
    b = oracle.dequantize(bc, bsc, 0.25)
    rows = np.unique(np.concatenate([np.arange(0, M, 97), np.arange(M - 60, M), [63, 64, 127, 128, 255, 256, 257]]))
    ref = oracle.gemm_f64(a[rows], b)
    na, nb = oracle.row_norms(a[rows]), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        y32 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_FP32, layout)
        check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
        y16 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_BF16, layout)
        check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
        assert torch.equal(y32.to(torch.bfloat16), y16)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits(rng.standard_normal((N, K)).astype(np.float32))
    a, b = oracle.bf16_to_f64(x[rows]), oracle.bf16_to_f64(w)
    y = mq.bf16_gemm(dev_bf16(x), dev_bf16(w), mq.MQ_OUT_BF16)
    check_gemm_bf16(host_bits(y[ridx]), oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b))


def test_two_column_ranges_in_two_tile_shapes():
    """M = 2040, N = 6096, K = 4096: 192 tiles of 256x256 would leave a quarter of the compute
    units idle, so the launcher gives the first 4096 columns to 256x128 tiles with K over wave
    pairs and the remaining 2000 to 128x128 tiles with K over the four waves (two launches on
    offset B, scale and output pointers).  Sampled rows, all columns: the seam at column 4096,
    the ragged last column tile and the guard band behind N must all be right."""
    rng = np.random.default_rng(77)
    M, N, K = 2040, 6096, 4096
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    a = oracle.dequantize(ac, asc, 0.5)
    b = oracle.dequantize(bc, bsc, 0.25)
    rows = np.unique(np.concatenate([np.arange(0, M, 173), np.arange(M - 40, M), [127, 128, 255, 256, 257, 1023, 1024]]))
    ref = oracle.gemm_f64(a[rows], b)
    na, nb = oracle.row_norms(a[rows]), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        ops = [ac, asc, bc, bsc]
        if layout == mq.MQ_LAYOUT_KTILE:
            ops[0], ops[1] = to_ktile(ac, asc)
            ops[2], ops[3] = to_ktile(bc, bsc)
        d = [dev_u8(v) for v in ops]
        aa, ba = dev_scalar(0.5), dev_scalar(0.25)
        ld = N + 24
        b32 = torch.full((M, ld), -7.0, dtype=torch.float32, device="cuda")
        b16 = torch.full((M, ld), -7.0, dtype=torch.bfloat16, device="cuda")
        y32 = mq.nvfp4_gemm(d[0], d[1], aa, d[2], d[3], ba, mq.MQ_OUT_FP32, b32[:, :N], layout=layout)
        y16 = mq.nvfp4_gemm(d[0], d[1], aa, d[2], d[3], ba, mq.MQ_OUT_BF16, b16[:, :N], layout=layout)
        torch.cuda.synchronize()
        check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
        check_gemm_bf16(host_bits(y16[ridx].contiguous()), ref, na, nb)
        assert torch.equal(y32.to(torch.bfloat16), y16)
        assert bool((b32[:, N:] == -7.0).all()) and bool((b16[:, N:] == -7.0).all())


# (M, N, K): ragged shapes with a long K on both sides of the launcher's choices.  With 256
# compute units: (1530, 6128, 4096) = 768 columns of 128x128 tiles + 5360 of 256x128 tiles;
# (3070, 6160, 4096) = 1024 columns of 128x128 + 5136 of 256x256; (3000, 6000, 4608) the same pair
# at another K; (2500, 9000, 4096) and (3300, 7000, 3072) = 256x128 + 256x256; (1300, 12000, 4096)
# = 128x128 + 256x256; (1800, 7360, 4992), (2900, 5008, 4096) one launch of 256x256 tiles;
# (911, 4128, 4800) of 256x128 tiles; (1190, 1888, 4224) of 128x128 tiles.
LAUNCH_SHAPES = [(1530, 6128, 4096), (3070, 6160, 4096), (3000, 6000, 4608), (2500, 9000, 4096),
                 (3300, 7000, 3072), (1300, 12000, 4096), (1800, 7360, 4992), (2900, 5008, 4096),
                 (911, 4128, 4800), (1190, 1888, 4224)]


@pytest.mark.parametrize("M,N,K", LAUNCH_SHAPES)
def test_ragged_shapes_across_launch_paths(M, N, K):
    """One tile shape or two column ranges in two shapes: sampled rows (tile seams, the ragged
    tail), all columns, both layouts, both output types."""
    rng = np.random.default_rng([M, N, K])
    print(f"\n[case] launch paths M={M} N={N} K={K}", flush=True)
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    a = oracle.dequantize(ac, asc, 0.5)
    b = oracle.dequantize(bc, bsc, 0.25)
    seams = np.arange(128, M, 128)
    rows = np.unique(np.concatenate([seams - 1, seams, rng.integers(0, M, 24), [0, M - 2, M - 1]]))
    rows = rows[(rows >= 0) & (rows < M)]
    ref = oracle.gemm_f64(a[rows], b)
    na, nb = oracle.row_norms(a[rows]), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        y32 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_FP32, layout)
        check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
        y16 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_BF16, layout)
        check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
        assert torch.equal(y32.to(torch.bfloat16), y16)


@pytest.mark.timeout(600)
def test_operand_larger_than_2_gib():
    """An activation operand of 2.3 GB: K-step and row offsets pass 2^31 in both layouts."""
    M, N, K = 320000, 256, 14336
    rng = np.random.default_rng(77)
    ac = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    asc = rng.integers(0x30, 0x40, size=(M, K // 16), dtype=np.uint8)
    bc, bsc = _rand_nvfp4(rng, N, K)
    rows = np.unique(np.concatenate([rng.integers(0, M, 48), [0, 1, 299593, 299594, M - 257, M - 256, M - 2, M - 1]]))
    a = oracle.dequantize(ac[rows], asc[rows], 0.5)
    b = oracle.dequantize(bc, bsc, 0.25)
    ref = oracle.gemm_f64(a, b)
    na, nb = oracle.row_norms(a), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        print(f"\n[case] layout={layout}", flush=True)
        A = (ac, asc) if layout == mq.MQ_LAYOUT_LINEAR else to_ktile(ac, asc)
        B = (bc, bsc) if layout == mq.MQ_LAYOUT_LINEAR else to_ktile(bc, bsc)
        acd, asd = dev_u8(A[0]), dev_u8(A[1])
        del A
        y = mq.nvfp4_gemm(acd, asd, dev_scalar(0.5), dev_u8(B[0]), dev_u8(B[1]), dev_scalar(0.25), mq.MQ_OUT_FP32,
                          None, layout)
        torch.cuda.synchronize()
        check_gemm_fp32(y[ridx].cpu().numpy(), ref, na, nb)
        del acd, asd, y
        torch.cuda.empty_cache()


@pytest.mark.timeout(600)
def test_bf16_operand_larger_than_4_gib():
    """A BF16 activation operand of 4.6 GB: row offsets pass 2^32 bytes.  The tiled kernel addresses
    rows relative to its tile, so it serves this shape like any other (no slow path)."""
    M, N, K = 160000, 256, 14336
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4321)
    x = torch.randn((M, K), dtype=torch.bfloat16, device="cuda", generator=gen)
    w = (torch.randn((N, K), dtype=torch.float32, device="cuda", generator=gen) * K ** -0.5).to(torch.bfloat16)
    rng = np.random.default_rng(78)
    first_past = (1 << 32) // (2 * K)      # first row that starts beyond 4 GiB
    rows = np.unique(np.concatenate([rng.integers(0, M, 40), [0, 1, 255, 256, first_past - 1, first_past,
                                                               first_past + 1, M - 257, M - 256, M - 2, M - 1]]))
    ridx = torch.from_numpy(rows).cuda()
    a = oracle.bf16_to_f64(host_bits(x[ridx]))
    b = oracle.bf16_to_f64(host_bits(w))
    ref = oracle.gemm_f64(a, b)
    na, nb = oracle.row_norms(a), oracle.row_norms(b)
    y32 = mq.bf16_gemm(x, w, mq.MQ_OUT_FP32)
    y16 = mq.bf16_gemm(x, w, mq.MQ_OUT_BF16)
    torch.cuda.synchronize()
    check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
    check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
    assert torch.equal(y32.to(torch.bfloat16), y16)
    del x, y32, y16
    torch.cuda.empty_cache()


@pytest.mark.parametrize("K", [64, 192, 448, 1280])
def test_four_way_split_k_path_with_ragged_edges(K):
    """256 workgroup tiles of 128x128 select the register-direct kernel with K split over its four
    waves (one K step: three parts are empty; three and seven: parts of unequal length)."""
    rng = np.random.default_rng(25 + K)
    M, N = 1000, 4000
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    a = oracle.dequantize(ac, asc, 0.5)
    b = oracle.dequantize(bc, bsc, 0.25)
    rows = np.unique(np.concatenate([np.arange(0, M, 37), np.arange(M - 40, M), [31, 32, 33, 63, 64, 95, 96, 127, 128]]))
    ref = oracle.gemm_f64(a[rows], b)
    na, nb = oracle.row_norms(a[rows]), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        y32 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_FP32, layout)
        check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
        y16 = _gpu_gemm(ac, asc, 0.5, bc, bsc, 0.25, mq.MQ_OUT_BF16, layout)
        check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
        assert torch.equal(y32.to(torch.bfloat16), y16)


def test_extreme_scales_subnormal_and_saturated():
    rng = np.random.default_rng(6)
    M, N, K = 70, 96, 256
    ac, asc = _rand_nvfp4(rng, M, K, 0x00, 0x7F)      # every E4M3 byte incl. subnormals and 448
    bc, bsc = _rand_nvfp4(rng, N, K, 0x00, 0x7F)
    a = oracle.dequantize(ac, asc, 1.0)
    b = oracle.dequantize(bc, bsc, 1.0)
    ref = oracle.gemm_f64(a, b)
    y32 = _gpu_gemm(ac, asc, 1.0, bc, bsc, 1.0, mq.MQ_OUT_FP32).cpu().numpy()
    check_gemm_fp32(y32, ref, oracle.row_norms(a), oracle.row_norms(b))


def test_closed_forms_and_single_products():
    K = 128
    ones_c = np.full((40, K // 2), 0x22, dtype=np.uint8)
    ones_s = np.full((40, K // 16), 0x38, dtype=np.uint8)
    y = _gpu_gemm(ones_c, ones_s, 0.25, ones_c[:32], ones_s[:32], 3.0, mq.MQ_OUT_FP32).cpu().numpy()
    assert (y == 0.25 * 3.0 * K).all()
    # one-hot: row c of A holds code c at k = 3 + 16*c % K ... every code pair, several scale pairs
    for sa, sb in [(0x38, 0x38), (0x01, 0x7E), (0x3D, 0x45), (0x07, 0x08), (0x7E, 0x7E)]:
        ac = np.zeros((16, K // 2), dtype=np.uint8)
        bc = np.zeros((16, K // 2), dtype=np.uint8)
        ac[:, 37] = np.arange(16) << 4      # element k = 75
        bc[:, 37] = np.arange(16) << 4
        asc = np.full((16, K // 16), sa, dtype=np.uint8)
        bsc = np.full((16, K // 16), sb, dtype=np.uint8)
        y = _gpu_gemm(ac, asc, 1.0, bc, bsc, 1.0, mq.MQ_OUT_FP32).cpu().numpy().astype(np.float64)
        ref = oracle.gemm_f64(oracle.dequantize(ac, asc, 1.0), oracle.dequantize(bc, bsc, 1.0))
        assert np.array_equal(y, ref)       # a single exact product per output


def test_k_position_one_hot_against_oracle():
    """An element at every k must meet exactly its partner (catches K-permutation mistakes)."""
    K = 192
    ac = np.zeros((K, K // 2), dtype=np.uint8)
    asc = np.full((K, K // 16), 0x38, dtype=np.uint8)
    for k in range(K):
        ac[k, k // 2] = 0x2 << (4 * (k & 1))          # A[k, k] = 1.0
    rng = np.random.default_rng(8)
    bc, bsc = _rand_nvfp4(rng, 48, K)
    b = oracle.dequantize(bc, bsc, 1.0)
    for layout in (mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE):
        y = _gpu_gemm(ac, asc, 1.0, bc, bsc, 1.0, mq.MQ_OUT_FP32, layout).cpu().numpy().astype(np.float64)
        assert np.array_equal(y, b.T)                 # Y[k, n] = B_hat[n, k]


def test_determinism_and_guard_band():
    rng = np.random.default_rng(9)
    M, N, K = 300, 264, 256
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    args = (dev_u8(ac), dev_u8(asc), dev_scalar(0.1), dev_u8(bc), dev_u8(bsc), dev_scalar(0.2))
    buf = torch.full((M + 9, N + 8), -7.0, dtype=torch.bfloat16, device="cuda")
    y = buf[:M, :N]
    mq.nvfp4_gemm(*args, mq.MQ_OUT_BF16, y)
    y2 = mq.nvfp4_gemm(*args, mq.MQ_OUT_BF16)
    ack, ask = to_ktile(ac, asc)
    bck, bsk = to_ktile(bc, bsc)
    y3 = mq.nvfp4_gemm(dev_u8(ack), dev_u8(ask), args[2], dev_u8(bck), dev_u8(bsk), args[5], mq.MQ_OUT_BF16,
                       layout=mq.MQ_LAYOUT_KTILE)
    assert torch.equal(y3, y2)            # same summation order in both layouts
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    assert (buf[M:] == -7.0).all() and (buf[:, N:] == -7.0).all()


def test_bf16_gemm_against_oracle():
    rng = np.random.default_rng(10)
    for M, N, K in [(256, 1024, 1024), (77, 200, 320), (5, 16, 40), (513, 264, 64),
                    # decode shapes (M <= 64, K % 128 == 0): the weight-streaming kernel
                    (1, 4096, 4096), (7, 272, 128), (16, 1000, 1024), (17, 48, 384), (33, 520, 2048),
                    (49, 16, 256), (64, 264, 14336),
                    # ... with two and four row tiles per wave (N >= 6144, N >= 24576), ragged N
                    (16, 6152, 256), (33, 8200, 384), (64, 8264, 256), (48, 9000, 128), (1, 8192, 1024),
                    (20, 4096, 2176), (5, 24584, 128), (40, 24640, 256), (64, 24576, 384)]:
        x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
        w = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
        a, b = oracle.bf16_to_f64(x), oracle.bf16_to_f64(w)
        ref = oracle.gemm_f64(a, b)
        na, nb = oracle.row_norms(a), oracle.row_norms(b)
        y32 = mq.bf16_gemm(dev_bf16(x), dev_bf16(w), mq.MQ_OUT_FP32).cpu().numpy()
        check_gemm_fp32(y32, ref, na, nb)
        y16 = host_bits(mq.bf16_gemm(dev_bf16(x), dev_bf16(w), mq.MQ_OUT_BF16))
        check_gemm_bf16(y16, ref, na, nb)


@pytest.mark.parametrize("K", [64, 192, 320])
def test_bf16_gemm_large_tiles_with_ragged_edges(K):
    """16 x 32 tiles of 256x256: the large-tile BF16 kernel, odd and even numbers of K steps."""
    rng = np.random.default_rng(40 + K)
    M, N = 256 * 15 + 77, 256 * 31 + 40
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
    rows = np.unique(np.concatenate([np.arange(0, M, 251), np.arange(M - 80, M), [127, 128, 255, 256, 257]]))
    a, b = oracle.bf16_to_f64(x[rows]), oracle.bf16_to_f64(w)
    ref = oracle.gemm_f64(a, b)
    na, nb = oracle.row_norms(a), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    xd, wd = dev_bf16(x), dev_bf16(w)
    buf = torch.full((M + 2, N + 8), -7.0, dtype=torch.float32, device="cuda")
    y32 = mq.bf16_gemm(xd, wd, mq.MQ_OUT_FP32, buf[:M, :N])
    y16 = mq.bf16_gemm(xd, wd, mq.MQ_OUT_BF16)
    torch.cuda.synchronize()
    check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
    check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
    assert torch.equal(y32.to(torch.bfloat16), y16)
    assert (buf[M:] == -7.0).all() and (buf[:, N:] == -7.0).all()


def test_gemm_errors_and_empty():
    from paper_2605_20315_amd import _lib
    lib = _lib.load()
    c = torch.zeros((4, 32), dtype=torch.uint8, device="cuda")
    s = torch.zeros((4, 4), dtype=torch.uint8, device="cuda")
    a = dev_scalar(1.0)
    y = torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    p = lambda t: t.data_ptr()
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 24, p(y), 8, 0, 0, st) == 2
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 2, 0, 0, st) == 2
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 8, 7, 0, st) == 4
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 8, 0, 3, st) == 4
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 48, p(y), 8, 0, 1, st) == 2
    assert lib.nvfp4_gemm(None, p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 8, 0, 0, st) == 1
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 12, 0, 0, st) == 3
    assert lib.nvfp4_gemm(p(c), p(s), p(a), p(c), p(s), p(a), 0, 4, 64, p(y), 8, 0, 0, st) == 0
    x = torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda")
    assert lib.bf16_gemm(p(x), 8, p(x), 8, 4, 4, 12, p(y), 8, 0, st) == 2
    assert lib.bf16_gemm(p(x), 8, p(x), 8, 4, 4, 8, p(y), 8, 0, st) == 0
    torch.cuda.synchronize()


def test_calls_follow_the_callers_stream():
    """Every entry point enqueues on the stream it is given: a chain issued on a side stream while
    the default stream is busy gives the same bytes as the same chain on the default stream."""
    rng = np.random.default_rng(77)
    M, K, N = 2048, 1024, 4096
    x = dev_bf16(wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)))
    w = dev_bf16(wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32)))
    aw = mq.nvfp4_global_scale(w)
    wc, ws = mq.nvfp4_quantize(w, aw, layout=mq.MQ_LAYOUT_KTILE)

    def chain():
        ax = mq.nvfp4_global_scale(x)
        xc, xs = mq.nvfp4_quantize(x, ax, layout=mq.MQ_LAYOUT_KTILE)
        return mq.nvfp4_gemm(xc, xs, ax, wc, ws, aw, mq.MQ_OUT_BF16, layout=mq.MQ_LAYOUT_KTILE), mq.bf16_gemm(x, w)
    ref4, ref16 = chain()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()            # default priority
    big = torch.empty((8192, 8192), dtype=torch.bfloat16, device="cuda")
    for _ in range(4):
        big.normal_()                     # keeps the default stream busy
    with torch.cuda.stream(side):
        y4, y16 = chain()
    side.synchronize()
    assert torch.equal(y4, ref4) and torch.equal(y16, ref16)
    torch.cuda.synchronize()


def test_chain_replays_from_a_hip_graph():
    """The entry points allocate nothing and never synchronise, so a dynamic-alpha NVFP4 linear
    (amax -> quantize -> GEMM) can be captured once and replayed on new inputs."""
    rng = np.random.default_rng(78)
    M, K, N = 2048, 1024, 4096
    mk = lambda: dev_bf16(wl.f32_to_bf16_bits((rng.standard_normal((M, K)) * rng.uniform(0.5, 4.0)).astype(np.float32)))
    w = dev_bf16(wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32)))
    aw = mq.nvfp4_global_scale(w)
    wc, ws = mq.nvfp4_quantize(w, aw, layout=mq.MQ_LAYOUT_KTILE)
    x = mk()
    ax = torch.empty(1, dtype=torch.float32, device="cuda")
    xc = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    xs = torch.empty((M, K // 16), dtype=torch.uint8, device="cuda")
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")

    def chain():
        mq.nvfp4_global_scale(x, ax)
        mq.nvfp4_quantize(x, ax, xc, xs, mq.MQ_LAYOUT_KTILE)
        mq.nvfp4_gemm(xc, xs, ax, wc, ws, aw, mq.MQ_OUT_BF16, y, mq.MQ_LAYOUT_KTILE)
    mq.mq_init()                           # one-time set-up of the device; no eager warm-up of the chain is needed
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for _ in range(3):
        x.copy_(mk())
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        chain()                            # eager, same input
        torch.cuda.synchronize()
        assert torch.equal(got, y)
