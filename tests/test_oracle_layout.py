"""Pins for the oracle's K-step-major byte permutation (the second byte order of an NVFP4 tensor
declared at mq_layout in include/mixquant.h).  CPU only.

Pins: a hand-worked example (tests/golden/ktile_layout.txt), the cases in which the permutation
must be the identity (one K step; one row), bijectivity and the inverse, the property the GEMM
relies on (the bytes of one K step of consecutive rows are one contiguous run), and one-hot
markers located with array reshapes instead of index arithmetic."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ktile_layout.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, spec = [p.strip() for p in line.split(":")]
            vals = []
            for part in spec.split():
                lo, hi = part.split("..")
                vals.extend(range(int(lo), int(hi) + 1))
            out[key] = np.array(vals, dtype=np.uint8)
    return out


def test_hand_worked_example():
    g = _golden()
    codes = g["codes_linear"].reshape(2, 64)
    scales = g["scales_linear"].reshape(2, 8)
    ck, sk = oracle.to_ktile(codes, scales)
    assert ck.reshape(-1).tolist() == g["codes_ktile"].tolist()
    assert sk.reshape(-1).tolist() == g["scales_ktile"].tolist()
    cl, sl = oracle.from_ktile(ck, sk)
    assert np.array_equal(cl, codes) and np.array_equal(sl, scales)


@pytest.mark.parametrize("rows,K", [(1, 64), (7, 64), (1, 640), (1, 4096)])
def test_identity_cases(rows, K):
    # one K step: the rows follow each other as in the canonical order; one row: the K steps do
    rng = np.random.default_rng([rows, K])
    codes = rng.integers(0, 256, (rows, K // 2)).astype(np.uint8)
    scales = rng.integers(0, 256, (rows, K // 16)).astype(np.uint8)
    ck, sk = oracle.to_ktile(codes, scales)
    assert np.array_equal(ck, codes) and np.array_equal(sk, scales)


@pytest.mark.parametrize("rows,K", [(2, 128), (5, 192), (33, 1024), (300, 448)])
def test_bijection_inverse_and_contiguous_k_steps(rows, K):
    T = K // 64
    n_c, n_s = rows * K // 2, rows * K // 16
    # distinct tags: 16-bit position split over two passes (low byte, high byte)
    pos_c, pos_s = np.arange(n_c), np.arange(n_s)
    where_c = np.zeros(n_c, dtype=np.int64)
    where_s = np.zeros(n_s, dtype=np.int64)
    for shift in (0, 8, 16):
        codes = ((pos_c >> shift) & 255).astype(np.uint8).reshape(rows, K // 2)
        scales = ((pos_s >> shift) & 255).astype(np.uint8).reshape(rows, K // 16)
        ck, sk = oracle.to_ktile(codes, scales)
        where_c |= ck.reshape(-1).astype(np.int64) << shift
        where_s |= sk.reshape(-1).astype(np.int64) << shift
        cl, sl = oracle.from_ktile(ck, sk)
        assert np.array_equal(cl, codes) and np.array_equal(sl, scales)
    # where_c[p] = canonical position of the byte stored at K-step-major position p
    assert np.array_equal(np.sort(where_c), pos_c) and np.array_equal(np.sort(where_s), pos_s)
    # the bytes of K step t are one contiguous run of rows * 32 (rows * 4) bytes, rows in order,
    # each row contributing its bytes [32 t, 32 t + 32) ([4 t, 4 t + 4)) in order
    lin_c = pos_c.reshape(rows, T, 32)
    lin_s = pos_s.reshape(rows, T, 4)
    for t in range(T):
        run_c = where_c[t * rows * 32:(t + 1) * rows * 32].reshape(rows, 32)
        run_s = where_s[t * rows * 4:(t + 1) * rows * 4].reshape(rows, 4)
        assert np.array_equal(run_c, lin_c[:, t, :])
        assert np.array_equal(run_s, lin_s[:, t, :])


def test_one_hot_markers():
    rows, K = 19, 320
    rng = np.random.default_rng(5)
    for _ in range(50):
        r, k = int(rng.integers(rows)), int(rng.integers(K))
        codes = np.zeros((rows, K // 2), dtype=np.uint8)
        scales = np.zeros((rows, K // 16), dtype=np.uint8)
        codes[r, k // 2] = 0xA5
        scales[r, k // 16] = 0x5A
        ck, sk = oracle.to_ktile(codes, scales)
        t3 = ck.reshape(K // 64, rows, 32)          # [K step][row][byte of the step]
        assert t3[k // 64, r, (k % 64) // 2] == 0xA5 and np.count_nonzero(ck) == 1
        s3 = sk.reshape(K // 64, rows, 4)
        assert s3[k // 64, r, (k % 64) // 16] == 0x5A and np.count_nonzero(sk) == 1


def test_rejects_k_not_multiple_of_64():
    with pytest.raises(AssertionError):
        oracle.to_ktile(np.zeros((2, 16), np.uint8), np.zeros((2, 2), np.uint8))
