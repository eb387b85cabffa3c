"""Pins for the oracle's quantizer (Eq. 2 then Eq. 1, Section 3.3).  CPU only.

Pins used: hand-worked blocks (tests/golden/nvfp4_blocks.txt), the exact-real reading of
Eq. 1-2 evaluated with rationals, the round-trip identity on exactly representable tensors,
the error bound implied by nearest rounding, the clipping invariant, and layout one-hots.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2605_20315_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "nvfp4_blocks.txt")
E2M1_GRID = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2),
             Fraction(3), Fraction(4), Fraction(6)]


def _bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            alpha, xs, sb, codes, packed = [p.strip() for p in line.split("|")]
            rows.append((float(alpha), [float(v) for v in xs.split()], int(sb, 16),
                         [int(c) for c in codes.split()], [int(b, 16) for b in packed.split()]))
    return rows


def test_golden_file_has_cases():
    assert len(_golden_rows()) >= 4


@pytest.mark.parametrize("case", _golden_rows())
def test_hand_worked_blocks(case):
    alpha, xs, sb, codes, packed = case
    x32 = np.array(xs, dtype=np.float32)
    bits = _bf16(x32)
    assert np.array_equal(wl.bf16_bits_to_f32(bits), x32), "fixture inputs must be BF16 values"
    got_codes, got_scales = oracle.quantize(bits.reshape(1, 16), alpha)
    assert got_scales.tolist() == [[sb]]
    assert got_codes.tolist() == [packed]
    unpacked = [(b >> (4 * j)) & 15 for b in got_codes[0] for j in (0, 1)]
    assert unpacked == codes


def _exact_nearest(v: Fraction, grid):
    best = None
    for i, g in enumerate(grid):
        d = abs(v - g)
        if best is None or d < best[0] or (d == best[0] and i % 2 == 0):
            best = (d, i)
    return best[1]


def _near_boundary(v: Fraction, grid, rel):
    """True when v lies within a relative distance rel of a midpoint between grid values."""
    for i in range(len(grid) - 1):
        mid = (grid[i] + grid[i + 1]) / 2
        if abs(v - mid) <= rel * mid:
            return True
    return False


@pytest.mark.parametrize("seed,alpha_mode", [(0, "amax"), (1, "amax"), (2, "pow2"), (3, "small")])
def test_quantizer_matches_exact_real_reading(seed, alpha_mode):
    """Eq. 1-2 over the reals (rationals), against the oracle's binary32 sequence.

    They may differ only where the exact argument sits within 2^-21 (relative) of a rounding
    boundary; everywhere else every scale byte and code must be identical."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((12, 64)).astype(np.float32)
    x[:, 5] *= 20
    x[3, :16] = 0
    x[4, 16:32] *= 1e-3
    bits = _bf16(x)
    if alpha_mode == "amax":
        alpha = float(oracle.global_scale(bits))
    elif alpha_mode == "pow2":
        alpha = 2.0 ** -6
    else:
        alpha = float(np.float32(3.1e-3))
    codes, scales = oracle.quantize(bits, alpha)
    e4m3 = [Fraction(oracle.e4m3_value(b)) for b in range(0x7F)]
    xv = wl.bf16_bits_to_f32(bits)
    A = Fraction(alpha)
    tol = Fraction(1, 2 ** 21)
    soft = 0
    for r in range(bits.shape[0]):
        for b in range(bits.shape[1] // 16):
            blk = [Fraction(float(v)) for v in xv[r, 16 * b:16 * b + 16]]
            arg = max(abs(v) for v in blk) / (A * 6)
            sb_exact = 0x7E if arg >= 448 else _exact_nearest(arg, e4m3)
            sb = int(scales[r, b])
            if sb != sb_exact:
                assert abs(sb - sb_exact) == 1 and _near_boundary(arg, e4m3, tol)
                soft += 1
            sigma = e4m3[sb]
            for i, v in enumerate(blk):
                byte = int(codes[r, 8 * b + i // 2])
                c = (byte >> 4) if i & 1 else (byte & 15)
                if sigma == 0:
                    assert (c & 7) == 0
                    continue
                y = abs(v) / (A * sigma)
                c_exact = 7 if y >= 6 else _exact_nearest(y, E2M1_GRID)
                if (c & 7) != c_exact:
                    assert abs((c & 7) - c_exact) == 1 and _near_boundary(y, E2M1_GRID, tol)
                    soft += 1
                assert (c >> 3) == (1 if np.signbit(xv[r, 16 * b + i]) else 0)
    assert soft <= 2


def test_round_trip_identity_on_representable_tensors():
    """With alpha a power of two, alpha*sigma*q is a BF16 value; quantizing it must return
    the same scale bytes and the same codes (codes of magnitude zero compare modulo sign)."""
    rng = np.random.default_rng(7)
    rows, K = 64, 256
    scales = rng.integers(0x08, 0x7F, size=(rows, K // 16)).astype(np.uint8)   # normal E4M3
    c = rng.integers(0, 16, size=(rows, K)).astype(np.uint8)
    c[:, ::16] = 7 | (c[:, ::16] & 8)          # one |q| = 6 per block pins the scale
    codes = (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)
    for alpha in (1.0, 2.0 ** -7, 2.0 ** 3):
        xhat = oracle.dequantize(codes, scales, alpha)
        bits = oracle.bf16_round(xhat)
        assert np.array_equal(oracle.bf16_to_f64(bits), xhat), "must be exact in BF16"
        codes2, scales2 = oracle.quantize(bits, alpha)
        assert np.array_equal(scales2, scales)
        c2 = np.stack([codes2 & 15, codes2 >> 4], axis=-1).reshape(rows, K)
        same = (c2 == c) | (((c2 & 7) == 0) & ((c & 7) == 0))
        assert same.all()


def test_dequantize_is_alpha_sigma_q():
    codes = np.tile(np.array([[0x21, 0xF7]], dtype=np.uint8), (1, 4))   # 16 elements
    scales = np.array([[0x3D]], dtype=np.uint8)                          # 1.625
    out = oracle.dequantize(codes, scales, 0.5)
    q = [0.5, 1.0, 6.0, -6.0] * 4
    assert out.tolist() == [[0.5 * 1.625 * v for v in q]]


def test_nibble_and_scale_order_one_hot():
    K = 64
    for k in range(K):
        x = np.zeros((2, K), dtype=np.float32)
        x[1, k] = 6.0
        codes, scales = oracle.quantize(_bf16(x), 1.0)
        exp_codes = np.zeros((2, K // 2), dtype=np.uint8)
        exp_codes[1, k // 2] = 7 << (4 * (k & 1))
        exp_scales = np.zeros((2, K // 16), dtype=np.uint8)
        exp_scales[1, k // 16] = 0x38
        assert np.array_equal(codes, exp_codes) and np.array_equal(scales, exp_scales)


def test_row_stride_is_honoured():
    rng = np.random.default_rng(11)
    big = _bf16(rng.standard_normal((8, 96)))
    view = big[:, 16:80]
    c1, s1 = oracle.quantize(view, 0.01)
    c2, s2 = oracle.quantize(np.ascontiguousarray(view), 0.01)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)


def test_zero_and_underflowing_blocks_give_signed_zero_codes():
    x = np.zeros((1, 48), dtype=np.float32)
    x[0, 16:32] = 1e-30
    x[0, 17] = -1e-30
    x[0, 32:48] = [2.0 ** -9 * 6] + [0.0] * 14 + [-0.0]
    codes, scales = oracle.quantize(_bf16(x), 1.0)
    assert scales.tolist() == [[0, 0, 1]]
    c = np.stack([codes & 15, codes >> 4], axis=-1).reshape(-1)
    assert c[:16].tolist() == [0] * 16
    assert c[16:32].tolist() == [0, 8] + [0] * 14
    assert c[32] == 7 and c[47] == 8


def test_subnormal_scales_and_the_two_to_minus_ten_tie():
    # Eq. 2 argument amax/6 at 2^-9, 1.5*2^-9 (tie -> even byte 2), 2^-10 (tie -> 0), just above.
    def scale_for(arg):
        x = np.zeros((1, 16), dtype=np.float32)
        x[0, 3] = np.float32(arg * 6)
        return int(oracle.quantize(_bf16(x), 1.0)[1][0, 0])
    assert scale_for(2.0 ** -9) == 1
    assert scale_for(1.5 * 2.0 ** -9) == 2
    assert scale_for(2.0 ** -10) == 0
    assert scale_for(2.0 ** -10 * 1.0078125) == 1


def test_block_amax_element_is_clipped_to_six_under_normal_unsaturated_scales():
    cfg = wl.configs()[0]
    bits = wl.activation(cfg, 0)
    alpha = oracle.global_scale(bits)
    codes, scales = oracle.quantize(bits, alpha)
    x = np.abs(wl.bf16_bits_to_f32(bits)).reshape(cfg.M, -1, 16)
    c = np.stack([codes & 15, codes >> 4], axis=-1).reshape(cfg.M, -1, 16) & 7
    arg = x.argmax(axis=2)
    top = np.take_along_axis(c, arg[..., None], axis=2)[..., 0]
    normal = (scales >= 0x08) & (scales < 0x7E)
    assert normal.mean() > 0.99
    assert (top[normal] == 7).all()
    assert scales.max() <= 0x7E and scales.max() >= 0x7D   # alpha = amax/2688 lands on 448


def test_quantization_error_is_within_half_a_grid_step():
    cfg = wl.configs()[0]
    bits = wl.activation(cfg, 0)
    alpha = oracle.global_scale(bits)
    codes, scales = oracle.quantize(bits, alpha)
    xhat = oracle.dequantize(codes, scales, alpha)
    x = oracle.bf16_to_f64(bits)
    sigma = np.array([oracle.e4m3_value(b) for b in range(256)])[scales]
    unit = np.repeat(float(alpha) * sigma, 16, axis=1)        # alpha * sigma per element
    ok = unit > 0
    y = np.abs(x[ok] / unit[ok])
    err = np.abs(x[ok] - xhat[ok]) / unit[ok]
    step = np.where(y < 2, 0.25, np.where(y < 4, 0.5, 1.0))
    unclipped = y <= 6
    assert (err[unclipped] <= step[unclipped] * (1 + 1e-6)).all()
    rel = np.linalg.norm(x - xhat) / np.linalg.norm(x)
    assert 0.05 < rel < 0.2      # a 4-bit format: roughly 10 % relative error


def test_global_scale_closed_form():
    x = np.zeros((3, 32), dtype=np.float32)
    assert oracle.global_scale(_bf16(x)) == np.float32(1.0)
    x[2, 7] = -10.0
    a = oracle.global_scale(_bf16(x))
    assert a == np.float32(10.0) / np.float32(2688.0)
    assert abs(float(a) - 0.003720238) < 1e-9
    _, scales = oracle.quantize(_bf16(x), a)
    assert scales[2, 0] == 0x7E


def test_rejects_k_not_multiple_of_16():
    import ctypes
    lib = oracle.ref._load()
    x = np.zeros((1, 24), dtype=np.uint16)
    out = np.zeros(64, dtype=np.uint8)
    rc = lib.nvfp4_ref_quantize(ctypes.c_void_p(x.ctypes.data), 1, 24, 24, 1.0,
                                ctypes.c_void_p(out.ctypes.data), ctypes.c_void_p(out.ctypes.data))
    assert rc == -1
