"""Pins for the two producer oracles (gated-MLP activation and RMS normalisation) that feed the
quantizer in the fused kernels.  Each check uses something other than the oracle's own formula:
an identity, an invariant, a closed form, or a different library routine."""
import numpy as np
import scipy.special

import oracle
from paper_2605_20315_amd import workloads as wl


def _bits(a):
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _vals(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def test_silu_mul_identities_and_library():
    rng = np.random.default_rng(1)
    g = _bits(rng.standard_normal((7, 96)) * 4.0)
    one = _bits(np.ones((7, 96)))
    pos = oracle.silu_mul_f64(np.concatenate([g, one], axis=1))
    neg = oracle.silu_mul_f64(np.concatenate([g ^ 0x8000, one], axis=1))   # silu(-g)
    gv = _vals(g)
    assert np.allclose(pos - neg, gv, rtol=0, atol=1e-14)                 # x*s(x) + x*s(-x) = x
    # (1 + tanh) cancels for negative arguments: absolute tolerance of a few double ulps of x
    assert np.allclose(pos, 0.5 * gv * (1.0 + np.tanh(0.5 * gv)), rtol=1e-13, atol=2e-15)
    assert np.allclose(pos, gv * scipy.special.expit(gv), rtol=1e-13, atol=1e-300)
    assert (np.sign(pos) == np.sign(gv)).all()


def test_silu_mul_halves_linearity_and_limits():
    rng = np.random.default_rng(2)
    g = _bits(rng.standard_normal((5, 64)) * 3.0)
    u = _bits(rng.standard_normal((5, 64)))
    base = oracle.silu_mul_f64(np.concatenate([g, u], axis=1))
    # linear in up: scaling up by 4 (exact in BF16) scales the result by exactly 4
    u4 = _bits(_vals(u) * 4.0)
    assert np.array_equal(oracle.silu_mul_f64(np.concatenate([g, u4], axis=1)), 4.0 * base)
    # the first half is the gate: a zero gate kills the product, a zero up does too, and the
    # halves are not interchangeable
    z = np.zeros_like(g)
    assert (oracle.silu_mul_f64(np.concatenate([z, u], axis=1)) == 0).all()
    assert (oracle.silu_mul_f64(np.concatenate([g, z], axis=1)) == 0).all()
    big, small = _bits(np.full((1, 16), 30.0)), _bits(np.full((1, 16), 0.125))
    assert np.allclose(oracle.silu_mul_f64(np.concatenate([big, small], axis=1)), 30.0 * 0.125, rtol=1e-12)
    swapped = oracle.silu_mul_f64(np.concatenate([small, big], axis=1))
    assert np.allclose(swapped, 0.125 / (1 + np.exp(-0.125)) * 30.0, rtol=1e-12) and swapped[0, 0] < 3.0
    # far negative gate: silu -> -0 without overflow trouble
    far = oracle.silu_mul_f64(np.concatenate([_bits(np.full((1, 16), -3.0e4)), small], axis=1))
    assert np.isfinite(far).all() and (np.abs(far) < 1e-300).all()
    # row stride: a view with a larger stride gives the same result
    wide = np.zeros((5, 200), dtype=np.uint16)
    wide[:, :128] = np.concatenate([g, u], axis=1)
    assert np.array_equal(oracle.silu_mul_f64(wide[:, :128]), base)


def test_rmsnorm_invariants_and_library():
    rng = np.random.default_rng(3)
    K = 160
    x = _bits(rng.standard_normal((6, K)) * np.exp(rng.standard_normal((6, 1))))
    w1 = _bits(np.ones(K))
    y = oracle.rmsnorm_f64(x, w1, 0.0)
    assert np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-13)             # unit RMS
    x8 = _bits(_vals(x) * 8.0)                                            # exact rescale
    assert np.allclose(oracle.rmsnorm_f64(x8, w1, 0.0), y, rtol=1e-15, atol=0)
    xv = _vals(x)
    assert np.allclose(y, xv * np.sqrt(K) / np.linalg.norm(xv, axis=1, keepdims=True), rtol=1e-13)
    # the weight multiplies per column
    w = _bits(rng.standard_normal(K))
    assert np.allclose(oracle.rmsnorm_f64(x, w, 0.0), y * _vals(w)[None, :], rtol=1e-15, atol=0)


def test_rmsnorm_eps_and_constant_rows():
    K = 64
    w = _bits(np.linspace(-2.0, 2.0, K))
    for c, eps in [(3.0, 0.0), (-0.5, 1e-6), (2.0, 0.25), (0.0, 1e-5)]:
        x = _bits(np.full((2, K), c))
        y = oracle.rmsnorm_f64(x, w, eps)
        expect = (c / np.sqrt(c * c + eps) if (c != 0 or eps > 0) else 0.0) * _vals(w)
        assert np.allclose(y, expect[None, :], rtol=1e-14, atol=0)
    # eps sits inside the square root and is added to the MEAN of squares, not the sum
    x = _bits(np.full((1, K), 1.0))
    y = oracle.rmsnorm_f64(x, _bits(np.ones(K)), 3.0)
    assert np.allclose(y, 0.5, rtol=1e-15)
    # row stride
    wide = np.zeros((3, 100), dtype=np.uint16)
    rng = np.random.default_rng(4)
    wide[:, :K] = _bits(rng.standard_normal((3, K)))
    dense = np.ascontiguousarray(wide[:, :K])
    assert np.array_equal(oracle.rmsnorm_f64(wide[:, :K], w, 1e-6), oracle.rmsnorm_f64(dense, w, 1e-6))
