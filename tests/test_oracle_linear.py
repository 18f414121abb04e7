"""Pins for the oracle's linear layer (Sec. 2: f^(i)(x^(i)) = x^(i) W^(i), the producer of the
partial sums that are compressed), and for linear-then-encode as the reference of a GEMM that
compresses in its epilogue.

Checked against integer arithmetic (exact), numpy's float64 matrix product and the half-ulp
bound of one rounding, the identity and selector matrices, and a brute-force loop on a tiny case.
"""
import numpy as np
import pytest

import oracle
from refmath import bits_to_f32, f32_to_bf16_bits_lib


def _bf16(a):
    return f32_to_bf16_bits_lib(np.asarray(a, np.float32))


def test_small_integers_are_exact():
    """Products and sums of small integers are exact in any precision: the result is the
    integer matrix product.  T, K, E all differ, so a transposed operand cannot pass."""
    rng = np.random.default_rng(3)
    T, K, E = 7, 24, 13
    Xi = rng.integers(-3, 4, (T, K))
    Wi = rng.integers(-3, 4, (E, K))
    Y = oracle.linear(_bf16(Xi), _bf16(Wi))
    want = Xi @ Wi.T                     # |.| <= 9 * 24 = 216: every integer up to 256 is a bf16 value
    assert np.array_equal(bits_to_f32(Y).astype(np.int64), want)


def test_one_rounding_of_the_float64_product():
    """Every output is within half a bf16 ulp of the float64 matrix product (one rounding, no
    intermediate binary32 step), and the magnitude output is the sum of |x w|."""
    rng = np.random.default_rng(5)
    T, K, E = 9, 200, 17
    X = _bf16(rng.standard_normal((T, K)) * 3)
    W = _bf16(rng.standard_normal((E, K)))
    Y, mag = oracle.linear(X, W, with_magnitude=True)
    X64, W64 = bits_to_f32(X).astype(np.float64), bits_to_f32(W).astype(np.float64)
    ref = X64 @ W64.T
    y = bits_to_f32(Y).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-300))) - 7)   # bf16: 8 significant bits
    # (numpy's product may differ from the exact sum by a few float64 ulps of the magnitudes)
    assert np.all(np.abs(y - ref) <= 0.5 * ulp + 1e-12 * (np.abs(X64) @ np.abs(W64).T))
    assert np.allclose(mag, np.abs(X64) @ np.abs(W64).T, rtol=1e-12)
    # and not a value rounded twice: where float32 rounding then bf16 rounding would differ
    # from one rounding, the oracle has the one-rounding value
    twice = f32_to_bf16_bits_lib(ref.astype(np.float32))
    differ = twice != Y
    for t, e in zip(*np.nonzero(differ)):
        assert abs(y[t, e] - ref[t, e]) <= abs(bits_to_f32(twice[t:t + 1, e:e + 1])[0, 0] - ref[t, e])


def test_ties_round_to_even():
    """x * w = 257 and 259 lie halfway between bf16 neighbours (256, 258, 260): one rounding to even."""
    X = _bf16([[1.0, 1.0], [1.0, 3.0]])
    W = _bf16([[256.0, 1.0]])          # row 0: 256 + 1 = 257 -> 256; row 1: 256 + 3 = 259 -> 260
    Y = bits_to_f32(oracle.linear(X, W))
    assert Y[0, 0] == 256.0 and Y[1, 0] == 260.0


def test_identity_and_selector_weights():
    rng = np.random.default_rng(7)
    T, K = 5, 16
    X = _bf16(rng.standard_normal((T, K)) * 10)
    assert np.array_equal(oracle.linear(X, _bf16(np.eye(K))), X)
    # output feature e takes input column sel[e], doubled
    sel = np.array([3, 0, 15, 7, 7], np.int64)
    W = np.zeros((sel.size, K), np.float32)
    W[np.arange(sel.size), sel] = 2.0
    got = bits_to_f32(oracle.linear(X, _bf16(W)))
    assert np.array_equal(got, 2.0 * bits_to_f32(X)[:, sel])


def test_brute_force_tiny():
    rng = np.random.default_rng(11)
    T, K, E = 2, 5, 3
    X = _bf16(rng.standard_normal((T, K)))
    W = _bf16(rng.standard_normal((E, K)))
    xf, wf = bits_to_f32(X), bits_to_f32(W)
    Y = bits_to_f32(oracle.linear(X, W))
    for t in range(T):
        for e in range(E):
            s = 0.0
            for k in range(K):
                s += float(xf[t, k]) * float(wf[e, k])
            assert abs(Y[t, e] - s) <= abs(s) * 2.0 ** -8


def test_threads_do_not_change_the_result():
    rng = np.random.default_rng(13)
    X = _bf16(rng.standard_normal((33, 64)))
    W = _bf16(rng.standard_normal((40, 64)))
    assert np.array_equal(oracle.linear(X, W, threads=1), oracle.linear(X, W, threads=4))


def test_bad_arguments():
    X = _bf16(np.zeros((2, 8)))
    W = _bf16(np.zeros((3, 9)))
    with pytest.raises(ValueError):
        oracle.linear(X, W)
