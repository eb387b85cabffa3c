"""Pins for the oracle's number formats and projections (Section 3.3: E2M1 elements, FP8 E4M3
block scales, Eq. 1's Pi_FP4 and Eq. 2's Pi_E4M3).  CPU only.

Each pin is something other than the oracle's own formula: the published value grids,
torch's independent FP8 / BF16 casts, exhaustive brute-force nearest searches written with
exact rationals, and structural properties (monotone, idempotent, ties to even).
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20315_amd import workloads as wl

E2M1_GRID = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_e2m1_all_16_codes_match_published_grid():
    for c in range(16):
        expect = E2M1_GRID[c & 7] * (-1.0 if c & 8 else 1.0)
        got = oracle.e2m1_value(c)
        assert got == expect and np.signbit(got) == bool(c & 8)


def test_e4m3_all_256_bytes_match_torch_float8():
    b = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = b.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for i in range(256):
        got = oracle.e4m3_value(i)
        if np.isnan(ref[i]):
            assert np.isnan(got) and (i & 0x7F) == 0x7F
        else:
            assert got == float(ref[i]), i
    assert oracle.e4m3_value(0x7E) == 448.0
    assert oracle.e4m3_value(0x01) == 2.0 ** -9
    assert oracle.e4m3_value(0x38) == 1.0


def test_e4m3_round_is_identity_on_grid_and_monotone():
    vals = [oracle.e4m3_value(b) for b in range(0x7F)]
    assert all(vals[i] < vals[i + 1] for i in range(0x7E))
    for b in range(0x7F):
        assert oracle.e4m3_round(vals[b]) == b
    xs = np.sort(np.abs(np.random.default_rng(1).standard_normal(20000)).astype(np.float32)
                 * np.float32(100.0))
    codes = [oracle.e4m3_round(float(x)) for x in xs]
    assert all(codes[i] <= codes[i + 1] for i in range(len(codes) - 1))


def test_e4m3_round_midpoints_tie_to_even_and_neighbours_do_not():
    for b in range(0x7E):
        lo, hi = oracle.e4m3_value(b), oracle.e4m3_value(b + 1)
        mid = np.float32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2  # representable in binary32
        even = b if b % 2 == 0 else b + 1
        assert oracle.e4m3_round(float(mid)) == even, b
        assert oracle.e4m3_round(float(np.nextafter(mid, np.float32(0)))) == b
        assert oracle.e4m3_round(float(np.nextafter(mid, np.float32(1e9)))) == b + 1


def test_e4m3_round_saturates_and_underflows():
    for v in [448.0, 449.0, 463.9, 464.0, 480.0, 1e9, float("inf")]:
        assert oracle.e4m3_round(v) == 0x7E
    assert oracle.e4m3_round(2.0 ** -10) == 0            # tie between 0 and 2^-9 -> even (0)
    assert oracle.e4m3_round(float(np.nextafter(np.float32(2.0 ** -10), np.float32(1)))) == 1
    assert oracle.e4m3_round(1e-30) == 0
    assert oracle.e4m3_round(0.0) == 0
    assert oracle.e4m3_round(1.5 * 2.0 ** -9) == 2       # tie between 0x01 and 0x02 -> even


def _nearest_exact(v: Fraction, grid):
    """Brute-force nearest grid index with ties to the even index; saturating."""
    best = None
    for i, g in enumerate(grid):
        d = abs(v - g)
        if best is None or d < best[0] or (d == best[0] and i % 2 == 0):
            best = (d, i)
    return best[1]


def test_e4m3_round_matches_exact_rational_brute_force():
    grid = [Fraction(oracle.e4m3_value(b)) for b in range(0x7F)]
    rng = np.random.default_rng(2)
    xs = np.concatenate([
        np.exp(rng.uniform(np.log(2.0 ** -12), np.log(600.0), 3000)),
        rng.uniform(0, 2.0 ** -5, 500),
    ]).astype(np.float32)
    for x in xs:
        assert oracle.e4m3_round(float(x)) == _nearest_exact(Fraction(float(x)), grid), x


def test_e4m3_round_matches_torch_cast_in_range():
    rng = np.random.default_rng(3)
    xs = np.exp(rng.uniform(np.log(2.0 ** -11), np.log(448.0), 20000)).astype(np.float32)
    ref = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_round(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(got, ref)


def test_fp4_round_exhaustive_over_all_bf16_inputs():
    """All 65 536 BF16 inputs against an independent numpy nearest search with explicit ties."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = wl.bf16_bits_to_f32(bits)
    finite = np.isfinite(vals)
    grid = np.array(E2M1_GRID)
    a = np.abs(vals.astype(np.float64))
    # lower neighbour index
    lo = np.clip(np.searchsorted(grid, a, side="right") - 1, 0, 7)
    hi = np.clip(lo + 1, 0, 7)
    dlo, dhi = a - grid[lo], grid[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    mag = np.where(hi == lo, lo, np.where(pick_hi, hi, lo))
    mag = np.where(a >= 6.0, 7, mag)
    expect = (mag | (np.signbit(vals).astype(np.int64) << 3)).astype(np.uint8)
    for i in np.nonzero(finite)[0]:
        assert oracle.fp4_round(float(vals[i])) == expect[i], hex(int(bits[i]))
    # infinities clip
    assert oracle.fp4_round(float("inf")) == 7 and oracle.fp4_round(float("-inf")) == 15


def test_fp4_round_named_ties_and_clipping():
    ties = {0.25: 0, 0.75: 2, 1.25: 2, 1.75: 4, 2.5: 4, 3.5: 6, 5.0: 6}
    for v, c in ties.items():
        assert oracle.fp4_round(v) == c
        assert oracle.fp4_round(-v) == (c | 8)
        up = float(np.nextafter(np.float32(v), np.float32(10)))
        dn = float(np.nextafter(np.float32(v), np.float32(0)))
        assert oracle.fp4_round(up) == E2M1_GRID.index(min(g for g in E2M1_GRID if g > v))
        assert oracle.fp4_round(dn) == E2M1_GRID.index(max(g for g in E2M1_GRID if g < v))
    for v in [6.0, 6.5, 100.0, 1e30]:
        assert oracle.fp4_round(v) == 7 and oracle.fp4_round(-v) == 15
    assert oracle.fp4_round(0.0) == 0 and oracle.fp4_round(-0.0) == 8
    assert oracle.fp4_round(-1e-30) == 8


def test_fp4_round_matches_exact_rational_brute_force():
    grid = [Fraction(g) for g in E2M1_GRID]
    rng = np.random.default_rng(4)
    xs = rng.uniform(-7, 7, 4000).astype(np.float32)
    for x in xs:
        expect = _nearest_exact(abs(Fraction(float(x))), grid) | (8 if x < 0 else 0)
        assert oracle.fp4_round(float(x)) == expect


def test_bf16_round_matches_torch_on_binary32_inputs_and_avoids_double_rounding():
    rng = np.random.default_rng(5)
    x = np.concatenate([
        rng.standard_normal(50000).astype(np.float32) * np.float32(50),
        np.float32(2.0) ** rng.integers(-140, 120, 2000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-45], dtype=np.float32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.bf16_round(x.astype(np.float64))
    assert np.array_equal(got, ref)
    # agrees with the generator's own BF16 rounding too
    assert np.array_equal(got, wl.f32_to_bf16_bits(x))
    # 1 + 2^-8 is the tie between 0x3F80 and 0x3F81; a hair above must round up even though
    # rounding through binary32 first would land on the tie and go down.
    v = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.bf16_round(np.array([v]))[0] == 0x3F81
    assert oracle.bf16_round(np.array([1.0 + 2.0 ** -8]))[0] == 0x3F80
    assert oracle.bf16_round(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82
    assert oracle.bf16_round(np.array([-v]))[0] == 0xBF81
