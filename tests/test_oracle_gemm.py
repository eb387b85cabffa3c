"""Pins for the oracle's block-scaled GEMM: Y = X_hat . W_hat^T with X_hat, W_hat the Eq. 1
dequantized operands (Section 3.3), evaluated in binary64.  CPU only.

Pins: closed forms, the exhaustive table of single products sigma_x*sigma_w*q_x*q_w, exact
rational brute force on tiny shapes, numpy's binary64 matmul, linearity in alpha and
invariance under a joint permutation of the 16-element blocks.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2605_20315_amd import workloads as wl

E2M1 = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def _rand_nvfp4(rng, rows, K):
    scales = rng.integers(0x20, 0x50, size=(rows, K // 16)).astype(np.uint8)
    codes = rng.integers(0, 256, size=(rows, K // 2)).astype(np.uint8)
    return codes, scales


def _gemm(ac, asc, aa, bc, bsc, ba):
    return oracle.gemm_f64(oracle.dequantize(ac, asc, aa), oracle.dequantize(bc, bsc, ba))


def test_all_ones_closed_form():
    M, N, K = 5, 7, 96
    ac = np.full((M, K // 2), 0x22, dtype=np.uint8)       # every element 1.0
    bc = np.full((N, K // 2), 0x22, dtype=np.uint8)
    asc = np.full((M, K // 16), 0x38, dtype=np.uint8)     # every scale 1.0
    bsc = np.full((N, K // 16), 0x38, dtype=np.uint8)
    y = _gemm(ac, asc, 0.25, bc, bsc, 3.0)
    assert (y == 0.25 * 3.0 * K).all()


def test_single_product_table_all_code_pairs_and_scale_sweep():
    K = 16
    sweep = [0x01, 0x07, 0x08, 0x30, 0x38, 0x3D, 0x45, 0x7E]
    for sa in sweep:
        for sb in sweep:
            ac = np.zeros((16, K // 2), dtype=np.uint8)
            bc = np.zeros((16, K // 2), dtype=np.uint8)
            for c in range(16):
                ac[c, 1] = c << 4        # element k = 3 of row c holds code c
                bc[c, 1] = c << 4
            asc = np.full((16, 1), sa, dtype=np.uint8)
            bsc = np.full((16, 1), sb, dtype=np.uint8)
            y = _gemm(ac, asc, 2.0, bc, bsc, 0.5)
            for i in range(16):
                for j in range(16):
                    qa = E2M1[i & 7] * (-1 if i & 8 else 1)
                    qb = E2M1[j & 7] * (-1 if j & 8 else 1)
                    expect = (oracle.e4m3_value(sa) * oracle.e4m3_value(sb)) * (qa * qb)
                    assert y[i, j] == expect


@pytest.mark.parametrize("shape", [(4, 4, 32), (3, 5, 48), (2, 3, 16)])
def test_exact_rational_brute_force(shape):
    M, N, K = shape
    rng = np.random.default_rng(sum(shape))
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    aa, ba = float(np.float32(0.0123)), float(np.float32(1.7e-3))
    y = _gemm(ac, asc, aa, bc, bsc, ba)

    def elems(codes, scales, alpha, r):
        out = []
        for k in range(K):
            byte = int(codes[r, k // 2])
            c = (byte >> 4) if k & 1 else (byte & 15)
            q = Fraction(E2M1[c & 7]) * (-1 if c & 8 else 1)
            out.append(Fraction(alpha) * Fraction(oracle.e4m3_value(int(scales[r, k // 16]))) * q)
        return out

    for m in range(M):
        xa = elems(ac, asc, aa, m)
        for n in range(N):
            xb = elems(bc, bsc, ba, n)
            exact = sum(p * q for p, q in zip(xa, xb))
            mag = sum(abs(p * q) for p, q in zip(xa, xb))
            assert abs(Fraction(float(y[m, n])) - exact) <= mag * Fraction(K, 2 ** 52)


def test_loop_gemm_matches_numpy_matmul():
    rng = np.random.default_rng(21)
    ac, asc = _rand_nvfp4(rng, 33, 256)
    bc, bsc = _rand_nvfp4(rng, 47, 256)
    a = oracle.dequantize(ac, asc, 0.01)
    b = oracle.dequantize(bc, bsc, 0.02)
    y = oracle.gemm_f64(a, b)
    ref = a @ b.T
    scale = np.abs(a) @ np.abs(b).T
    assert (np.abs(y - ref) <= 1e-13 * scale).all()
    # a transposed-operand mistake would show on a non-square case
    assert y.shape == (33, 47)


def test_bf16_reference_gemm_matches_numpy():
    rng = np.random.default_rng(22)
    x = wl.f32_to_bf16_bits(rng.standard_normal((19, 80)).astype(np.float32))
    w = wl.f32_to_bf16_bits(rng.standard_normal((23, 80)).astype(np.float32))
    xf, wf = oracle.bf16_to_f64(x), oracle.bf16_to_f64(w)
    assert np.array_equal(xf, wl.bf16_bits_to_f32(x).astype(np.float64))
    y = oracle.gemm_f64(xf, wf)
    ref = xf @ wf.T
    assert np.allclose(y, ref, rtol=0, atol=1e-12)


def test_linearity_in_alpha_and_block_permutation_invariance():
    rng = np.random.default_rng(23)
    M, N, K = 6, 9, 128
    ac, asc = _rand_nvfp4(rng, M, K)
    bc, bsc = _rand_nvfp4(rng, N, K)
    y1 = _gemm(ac, asc, 1.0, bc, bsc, 1.0)
    y2 = _gemm(ac, asc, 0.5, bc, bsc, 4.0)
    assert np.array_equal(y2, 2.0 * y1)
    perm = rng.permutation(K // 16)
    acp = ac.reshape(M, K // 16, 8)[:, perm].reshape(M, K // 2)
    bcp = bc.reshape(N, K // 16, 8)[:, perm].reshape(N, K // 2)
    y3 = _gemm(acp, asc[:, perm], 1.0, bcp, bsc[:, perm], 1.0)
    scale = np.abs(oracle.dequantize(ac, asc, 1.0)) @ np.abs(oracle.dequantize(bc, bsc, 1.0)).T
    assert (np.abs(y3 - y1) <= 1e-13 * scale).all()


def test_row_norms():
    a = np.array([[3.0, 4.0, 0.0], [1.0, 2.0, 2.0]])
    assert oracle.row_norms(a).tolist() == [5.0, 3.0]


def test_tiny_config_end_to_end_quantization_error_is_small_but_nonzero():
    """Sanity of the whole chain on the smallest workload: the NVFP4 product is close to the
    BF16 product (a few percent of ||row||.||col||), not equal to it."""
    cfg = wl.configs()[0]
    x, w = wl.activation(cfg, 0), wl.weight(cfg, 0)
    ax, aw = oracle.global_scale(x), oracle.global_scale(w)
    xc, xs = oracle.quantize(x, ax)
    wc, ws = oracle.quantize(w, aw)
    xh, wh = oracle.dequantize(xc[:32], xs[:32], ax), oracle.dequantize(wc, ws, aw)
    y = oracle.gemm_f64(xh, wh)
    yb = oracle.gemm_f64(oracle.bf16_to_f64(x[:32]), oracle.bf16_to_f64(w))
    bound = np.outer(oracle.row_norms(xh), oracle.row_norms(wh))
    rel = np.abs(y - yb) / bound
    assert 1e-4 < rel.max() < 0.1
