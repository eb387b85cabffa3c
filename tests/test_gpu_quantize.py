"""GPU parity: nvfp4_quantize / nvfp4_global_scale (C ABI, HIP kernels) against the CPU oracle.
The bar is bit-exact: every code byte and every scale byte (Eq. 1-2, Section 3.3)."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import workloads as wl

from _gpu_util import dev_bf16, dev_scalar, to_ktile

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "nvfp4_blocks.txt")


def _bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _run(bits: np.ndarray, alpha):
    xd = dev_bf16(bits)
    codes, scales = mq.nvfp4_quantize(xd, dev_scalar(alpha))
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy()


def _assert_same(bits, alpha):
    c_ref, s_ref = oracle.quantize(bits, alpha)
    c, s = _run(bits, alpha)
    assert np.array_equal(s, s_ref), f"{(s != s_ref).sum()} scale bytes differ"
    assert np.array_equal(c, c_ref), f"{(c != c_ref).sum()} code bytes differ"
    if bits.shape[1] % 64 == 0:      # the K-step-major layout holds the same bytes, permuted
        ck, sk = mq.nvfp4_quantize(dev_bf16(bits), dev_scalar(alpha), layout=mq.MQ_LAYOUT_KTILE)
        ck_ref, sk_ref = to_ktile(c_ref, s_ref)
        assert np.array_equal(sk.cpu().numpy(), sk_ref) and np.array_equal(ck.cpu().numpy(), ck_ref)


def test_tiny_config_bit_exact_and_global_scale():
    cfg = wl.configs()[0]
    for bits in (wl.activation(cfg, 0), wl.weight(cfg, 0)):
        alpha_ref = oracle.global_scale(bits)
        alpha = mq.nvfp4_global_scale(dev_bf16(bits))
        assert np.float32(alpha.item()) == alpha_ref
        _assert_same(bits, alpha_ref)


def test_golden_blocks():
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            alpha, xs, sb, _, packed = [p.strip() for p in line.split("|")]
            bits = _bf16([float(v) for v in xs.split()]).reshape(1, 16)
            c, s = _run(bits, float(alpha))
            assert s.tolist() == [[int(sb, 16)]]
            assert c.tolist() == [[int(b, 16) for b in packed.split()]]


def test_adversarial_blocks():
    rng = np.random.default_rng(0)
    rows = []
    ties = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    # every tie and its BF16 neighbours, both signs, with a 6 pinning sigma = 1
    for t in ties:
        up = wl.bf16_bits_to_f32(_bf16([t]) + np.uint16(1))[0]
        dn = wl.bf16_bits_to_f32(_bf16([t]) - np.uint16(1))[0]
        rows.append([6.0, t, -t, up, -up, dn, -dn, 0.0, -0.0, 1e-30, -1e-30, 0.5, 1.5, 3.0, 4.0, -6.0])
    rows.append([0.0] * 16)
    rows.append([-0.0] * 16)
    rows.append([1e-30] * 8 + [-1e-30] * 8)
    for arg in (2.0 ** -9, 1.5 * 2.0 ** -9, 2.0 ** -10, 2.0 ** -10 * 1.0078125, 2.0 ** -6, 2.0 ** -7 * 1.9375):
        rows.append([arg * 6] + [arg * v for v in rng.uniform(-6, 6, 15)])
    rows.append([3e38, -3e38] + [1.0] * 14)
    x = np.array(rows, dtype=np.float32)
    bits = _bf16(x)
    for alpha in (1.0, 0.5, 2.0 ** -7, float(np.float32(3.3e-3)), 1e-4, 7.0):
        _assert_same(bits, alpha)      # small alphas saturate the block scale at 448 and clip
    _assert_same(bits, oracle.global_scale(bits))


def test_all_bf16_magnitudes_with_many_scales():
    """Every finite BF16 value appears in some block, under several tensor scales, so that
    the multiply-then-round path meets arguments with long mantissas near every boundary."""
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    allbits = allbits[np.isfinite(wl.bf16_bits_to_f32(allbits))]
    rng = np.random.default_rng(1)
    pad = (-len(allbits)) % 16
    bits = np.concatenate([allbits, allbits[:pad]])
    bits = bits[rng.permutation(len(bits))].reshape(-1, 16)
    sel = np.abs(wl.bf16_bits_to_f32(bits)).max(axis=1) < 1e30     # keep alpha*sigma in range
    bits = np.ascontiguousarray(bits[sel])
    for alpha in (1.0, float(np.float32(1.7)), float(np.float32(1e5)), float(np.float32(1e20))):
        _assert_same(bits, alpha)
    srt = np.sort(allbits[wl.bf16_bits_to_f32(allbits) > 0])
    srt = srt[: len(srt) // 16 * 16].reshape(-1, 16)             # blocks of similar magnitude
    for alpha in (1.0, float(np.float32(0.37)), float(np.float32(2.9e-2))):
        _assert_same(srt, alpha)


def test_random_tensors_many_shapes_and_strides():
    rng = np.random.default_rng(2)
    for rows, K in [(1, 16), (3, 48), (17, 1008), (255, 4096), (300, 272), (64, 14336), (1, 64), (37, 192),
                    (16, 256), (513, 320)]:
        x = rng.standard_normal((rows, K)).astype(np.float32) * np.exp(rng.standard_normal((rows, 1))).astype(np.float32)
        bits = _bf16(x)
        _assert_same(bits, oracle.global_scale(bits))
    # a row stride larger than K
    big = _bf16(rng.standard_normal((37, 640)))
    view = big[:, 64:576]
    alpha = 0.004
    xd = dev_bf16(big)[:, 64:576]
    assert xd.stride(0) == 640
    codes, scales = mq.nvfp4_quantize(xd, dev_scalar(alpha))
    c_ref, s_ref = oracle.quantize(view, alpha)
    assert np.array_equal(codes.cpu().numpy(), c_ref) and np.array_equal(scales.cpu().numpy(), s_ref)
    a = mq.nvfp4_global_scale(xd)
    assert np.float32(a.item()) == oracle.global_scale(np.ascontiguousarray(view))


def test_outputs_beyond_the_tensor_are_untouched_and_empty_input_is_a_noop():
    rng = np.random.default_rng(3)
    rows, K = 77, 208
    bits = _bf16(rng.standard_normal((rows, K)))
    guard = 4096
    codes = torch.full((rows * K // 2 + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    scales = torch.full((rows * K // 16 + guard,), 0x5A, dtype=torch.uint8, device="cuda")
    mq.nvfp4_quantize(dev_bf16(bits), dev_scalar(0.01), codes[: rows * K // 2].view(rows, K // 2),
                      scales[: rows * K // 16].view(rows, K // 16))
    torch.cuda.synchronize()
    assert (codes[rows * K // 2:] == 0xA5).all() and (scales[rows * K // 16:] == 0x5A).all()
    c_ref, s_ref = oracle.quantize(bits, 0.01)
    assert np.array_equal(codes[: rows * K // 2].cpu().numpy().reshape(rows, -1), c_ref)
    assert np.array_equal(scales[: rows * K // 16].cpu().numpy().reshape(rows, -1), s_ref)
    codes.fill_(0xA5)
    scales.fill_(0x5A)
    K2 = 192
    bits2 = _bf16(rng.standard_normal((rows, K2)))
    mq.nvfp4_quantize(dev_bf16(bits2), dev_scalar(0.01), codes[: rows * K2 // 2].view(rows, K2 // 2),
                      scales[: rows * K2 // 16].view(rows, K2 // 16), mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    assert (codes[rows * K2 // 2:] == 0xA5).all() and (scales[rows * K2 // 16:] == 0x5A).all()
    ck_ref, sk_ref = to_ktile(*oracle.quantize(bits2, 0.01))
    assert np.array_equal(codes[: rows * K2 // 2].cpu().numpy().reshape(rows, -1), ck_ref)
    assert np.array_equal(scales[: rows * K2 // 16].cpu().numpy().reshape(rows, -1), sk_ref)
    empty = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    c, s = mq.nvfp4_quantize(empty, dev_scalar(1.0))
    assert c.shape == (0, 32) and s.shape == (0, 4)
    assert mq.nvfp4_global_scale(empty).item() == 1.0
    zeros = torch.zeros((5, 64), dtype=torch.bfloat16, device="cuda")
    assert mq.nvfp4_global_scale(zeros).item() == 1.0


def test_quantizer_is_deterministic():
    cfg = wl.configs()[0]
    xd = dev_bf16(wl.activation(cfg, 0))
    alpha = mq.nvfp4_global_scale(xd)
    c1, s1 = mq.nvfp4_quantize(xd, alpha)
    c2, s2 = mq.nvfp4_quantize(xd, alpha)
    assert torch.equal(c1, c2) and torch.equal(s1, s2)


def test_errors_are_reported_not_launched():
    from paper_2605_20315_amd import _lib
    lib = _lib.load()
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    a = dev_scalar(1.0)
    c = torch.zeros((4, 32), dtype=torch.uint8, device="cuda")
    s = torch.zeros((4, 4), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    assert lib.nvfp4_quantize(x.data_ptr(), 4, 24, 24, a.data_ptr(), c.data_ptr(), s.data_ptr(), 0, st) == 2
    assert lib.nvfp4_quantize(x.data_ptr(), 4, 64, 32, a.data_ptr(), c.data_ptr(), s.data_ptr(), 0, st) == 2
    assert lib.nvfp4_quantize(None, 4, 64, 64, a.data_ptr(), c.data_ptr(), s.data_ptr(), 0, st) == 1
    assert lib.nvfp4_quantize(x.data_ptr() + 2, 3, 64, 64, a.data_ptr(), c.data_ptr(), s.data_ptr(), 0, st) == 3
    assert lib.nvfp4_quantize(x.data_ptr(), 4, 64, 68, a.data_ptr(), c.data_ptr(), s.data_ptr(), 0, st) == 3
    assert lib.nvfp4_quantize(x.data_ptr(), 4, 48, 48, a.data_ptr(), c.data_ptr(), s.data_ptr(), 1, st) == 2
    assert lib.nvfp4_quantize(x.data_ptr(), 4, 64, 64, a.data_ptr(), c.data_ptr(), s.data_ptr(), 9, st) == 4
    with pytest.raises(mq.MixQuantError):
        mq.nvfp4_quantize(torch.zeros((4, 64), dtype=torch.bfloat16), torch.ones(1))


def test_relayout_is_the_documented_permutation_and_round_trips():
    rng = np.random.default_rng(12)
    for rows, K in [(1, 64), (77, 192), (300, 1024), (1024, 4096)]:
        bits = _bf16(rng.standard_normal((rows, K)))
        c_ref, s_ref = oracle.quantize(bits, 0.01)
        ck_ref, sk_ref = to_ktile(c_ref, s_ref)
        cd, sd = torch.from_numpy(c_ref).cuda(), torch.from_numpy(s_ref).cuda()
        ck, sk = mq.nvfp4_relayout(cd, sd, mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_KTILE)
        assert np.array_equal(ck.cpu().numpy(), ck_ref) and np.array_equal(sk.cpu().numpy(), sk_ref)
        cl, sl = mq.nvfp4_relayout(ck, sk, mq.MQ_LAYOUT_KTILE, mq.MQ_LAYOUT_LINEAR)
        assert torch.equal(cl, cd) and torch.equal(sl, sd)
    with pytest.raises(mq.MixQuantError):
        mq.nvfp4_relayout(cd, sd, mq.MQ_LAYOUT_LINEAR, mq.MQ_LAYOUT_LINEAR)
