"""Pins for the oracle's static symmetric mode (the paper's own quantiser, Sec. 3).

The paper fixes: static parameters per device and per feature from calibration; the
symmetric range R = 2*max(-m, M); everything that is not kept in BF16 is symmetrically
quantised to Int4; only codes and the BF16 features travel (4 + 12k/E bits per value,
Sec. 1 and 4).  The step (R/15), the code set (-8..7) and the nibble on the wire (code + 8)
are this build's reading.  Everything is checked against definitions written independently
of the oracle: a float64 search over the 16 levels, closed forms, numpy sums, and a
hand-worked example.
"""
import os

import numpy as np
import pytest

import oracle
from refmath import (bits_to_f32, compaction, f32_to_bf16_bits_lib, f32_vals_to_bits,
                     payload_bits, unpack_codes)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "static_worked_example.txt")


def test_worked_example():
    spec = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            key, *rest = line.split()
            spec[key] = rest
    E = int(spec["E"][0])
    idx = np.array([int(v) for v in spec["idx"]], np.int32)
    m = np.array([[float(v) for v in spec["m"]]], np.float32)
    M = np.array([[float(v) for v in spec["M"]]], np.float32)
    step, inv = oracle.static_params(m, M)
    comp = compaction(idx, E)
    assert step[0, comp].tolist() == [float(v) for v in spec["expect_step"]]
    Y = f32_vals_to_bits(np.array([[float(v) for v in spec["row"]]], np.float32))
    msg = oracle.encode_static(Y, idx, inv[0])
    assert bits_to_f32(msg.outl)[0].tolist() == [float(v) for v in spec["expect_outl"]]
    assert msg.codes[0].tolist() == [int(v, 16) for v in spec["expect_codes"]]
    xh = oracle.decode_reduce_static([msg], idx, step, oracle.ACC_FP32, out_fp32=True)
    assert xh[0].tolist() == [float(v) for v in spec["expect_dequant"]]
    step2 = np.concatenate([step, step])
    for accum in (oracle.ACC_FP32, oracle.ACC_BF16):
        s2 = oracle.decode_reduce_static([msg, msg], idx, step2, accum, out_fp32=False)
        assert bits_to_f32(s2)[0].tolist() == [float(v) for v in spec["expect_sum2"]]


def test_static_params_closed_form():
    """R = 2*max(-m, M) (Sec. 3), step = R/15, inv = 1/step; a vanishing range gives 0, 0."""
    rng = np.random.default_rng(1)
    m = -np.abs(rng.standard_normal((3, 500))).astype(np.float32) * 10
    M = np.abs(rng.standard_normal((3, 500))).astype(np.float32) * 10
    m[0, :5] = [1.0, 2.0, 0.0, -0.0, 3.0]      # one-signed and empty columns
    M[0, :5] = [4.0, 1.0, 0.0, 0.0, 3.0]
    m[1, :3] = [-5.0, -1e-31, -2.0]
    M[1, :3] = [-1.0, 1e-31, -3.0]             # all-negative column; range below the threshold; M < m
    step, inv = oracle.static_params(m, M)
    R = 2.0 * np.maximum(-m.astype(np.float64), M.astype(np.float64))
    live = R / 15.0 >= 1e-30
    assert np.all(step[~live] == 0) and np.all(inv[~live] == 0)
    assert np.all(np.abs(step[live] * 15.0 - R[live]) <= R[live] * 2.0 ** -22)
    assert np.all(np.abs(step[live].astype(np.float64) * inv[live] - 1.0) <= 2.0 ** -22)
    assert step[0, 0] == np.float32(8.0) / np.float32(15.0)      # m = 1, M = 4: R = 8
    assert step[0, 1] == np.float32(2.0) / np.float32(15.0)      # m = 2, M = 1: max(-2, 1) = 1
    assert step[0, 2] == 0 and step[0, 3] == 0                   # zero ranges, either sign of zero
    assert step[1, 0] == np.float32(10.0) / np.float32(15.0)     # m = -5, M = -1: max(5, -1) = 5
    assert step[1, 1] == 0                                       # vanishing range


def _check(Y, idx, step, inv, msg):
    T, E = Y.shape
    r = E - idx.size
    comp = compaction(idx, E)
    assert np.array_equal(msg.outl, Y[:, idx])                    # BF16 features verbatim
    if r == 0:
        return
    x = bits_to_f32(Y)[:, comp].astype(np.float64)
    nib, pad = unpack_codes(msg.codes, r)
    assert np.all(pad == 0)
    q = nib.astype(np.int64) - 8
    s = step[comp].astype(np.float64)[None, :]
    # brute force: the chosen level is the nearest of the 16 levels -8..7 times step
    levels = np.arange(-8, 8)[None, None, :] * s[..., None]
    dist = np.abs(x[..., None] - levels)
    chosen = np.take_along_axis(dist, (q + 8)[..., None], -1)[..., 0]
    # a tie region: the encoder multiplies by a rounded reciprocal
    assert np.all(chosen <= dist.min(-1) + s * 2.0 ** -16)
    dead = (s == 0) & np.ones_like(x, bool)
    assert np.all(q[dead] == 0)
    # inside the representable range the error is at most half a step; outside it saturates
    inside = (x >= -8.0 * s) & (x <= 7.0 * s) & ~dead
    err = np.abs(q * s - x)
    assert np.all(err[inside] <= 0.5 * s.repeat(T, 0)[inside] * (1 + 2.0 ** -18))
    assert np.all(q[(x > 7.5 * s * (1 + 2.0 ** -20)) & ~dead] == 7)
    assert np.all(q[(x < -8.5 * s * (1 + 2.0 ** -20)) & ~dead] == -8)


@pytest.mark.parametrize("E,k,T", [(64, 0, 5), (96, 3, 4), (105, 8, 3), (520, 9, 3), (32, 32, 2), (17, 16, 3)])
def test_brute_force_shapes(E, k, T):
    rng = np.random.default_rng(E * 10 + k)
    x = rng.standard_normal((T, E)).astype(np.float32) * 3
    x[:, ::5] *= 30                                  # values far outside the calibrated range
    Y = f32_to_bf16_bits_lib(x)
    m = -np.abs(rng.standard_normal((1, E))).astype(np.float32) * 4 - 0.5
    M = np.abs(rng.standard_normal((1, E))).astype(np.float32) * 4 + 0.5
    m[0, 1::9] = 0
    M[0, 1::9] = 0                                   # dead features
    step, inv = oracle.static_params(m, M)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    msg = oracle.encode_static(Y, idx, inv[0])
    _check(Y, idx, step[0], inv[0], msg)


def test_grid_inputs_round_trip_exactly():
    """Inputs on the code grid of a power-of-two step come back exactly, for every code."""
    E, T = 64, 16
    step = np.full((1, E), 0.25, np.float32)
    m = -step * 7.5
    M = step * 7.5                                  # R = 15 * step
    got_step, inv = oracle.static_params(m, M)
    assert np.array_equal(got_step, step)
    q = (np.arange(T * E).reshape(T, E) % 16) - 8
    Y = f32_vals_to_bits((q * 0.25).astype(np.float32))
    idx = np.zeros(0, np.int32)
    msg = oracle.encode_static(Y, idx, inv[0])
    nib, _ = unpack_codes(msg.codes, E)
    assert np.array_equal(nib.astype(np.int64) - 8, q)
    xh = oracle.decode_reduce_static([msg], idx, step, oracle.ACC_FP32, out_fp32=True)
    assert np.array_equal(xh, q * 0.25)


def test_sum_over_devices_matches_numpy():
    """decode_reduce = sum over devices of code * step (and of the BF16 features), in order."""
    rng = np.random.default_rng(3)
    N, T, E, k = 5, 6, 128, 4
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    m = -np.abs(rng.standard_normal((N, E))).astype(np.float32) * 3 - 1
    M = np.abs(rng.standard_normal((N, E))).astype(np.float32) * 3 + 1
    step, inv = oracle.static_params(m, M)
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 2) for _ in range(N)]
    msgs = [oracle.encode_static(Ys[i], idx, inv[i]) for i in range(N)]
    comp = compaction(idx, E)
    want = np.zeros((T, E), np.float32)
    for i in range(N):                       # fp32 chain in device order
        nib, _ = unpack_codes(msgs[i].codes, E - k)
        term = np.zeros((T, E), np.float32)
        term[:, comp] = (nib.astype(np.float32) - np.float32(8)) * step[i][comp][None, :]
        term[:, idx] = bits_to_f32(msgs[i].outl)
        want = term if i == 0 else (want + term).astype(np.float32)
    got = oracle.decode_reduce_static(msgs, idx, step, oracle.ACC_FP32, out_fp32=True)
    assert np.array_equal(got, want)
    got16 = oracle.decode_reduce_static(msgs, idx, step, oracle.ACC_FP32, out_fp32=False)
    assert np.array_equal(got16, f32_to_bf16_bits_lib(want))
    # bf16 chain: every term and partial sum through the library's bf16 conversion
    acc = None
    for i in range(N):
        nib, _ = unpack_codes(msgs[i].codes, E - k)
        term = np.zeros((T, E), np.float32)
        term[:, comp] = (nib.astype(np.float32) - np.float32(8)) * step[i][comp][None, :]
        term[:, idx] = bits_to_f32(msgs[i].outl)
        term = bits_to_f32(f32_to_bf16_bits_lib(term))
        acc = term if acc is None else bits_to_f32(f32_to_bf16_bits_lib((acc + term).astype(np.float32)))
    got_b = oracle.decode_reduce_static(msgs, idx, step, oracle.ACC_BF16, out_fp32=False)
    assert np.array_equal(bits_to_f32(got_b), acc)


def test_every_feature_selected_is_a_plain_sum():
    rng = np.random.default_rng(4)
    N, T, E = 3, 4, 24
    idx = np.arange(E, dtype=np.int32)
    step = np.ones((N, E), np.float32)
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32)) for _ in range(N)]
    msgs = [oracle.encode_static(Y, idx, np.ones(E, np.float32)) for Y in Ys]
    assert all(mg.codes.shape == (T, 0) for mg in msgs)
    got = oracle.decode_reduce_static(msgs, idx, step, oracle.ACC_FP32, out_fp32=True)
    want = bits_to_f32(Ys[0])
    for Y in Ys[1:]:
        want = (want + bits_to_f32(Y)).astype(np.float32)
    assert np.array_equal(got, want)


def test_bits_per_value_is_the_papers_count():
    """Nothing but codes and BF16 features travels: 4 + 12k/E bits (Sec. 1, 4): 4.1875 at k = E/64."""
    for E in (4608, 5120, 8192):
        k = E // 64
        Y = np.zeros((1, E), np.uint16)
        msg = oracle.encode_static(Y, np.arange(k, dtype=np.int32), np.ones(E, np.float32))
        bits = 8.0 * (msg.codes.nbytes + msg.outl.nbytes) / E
        assert bits == payload_bits(E, k) == 4.1875


def test_quantisation_error_is_uniform_inside_the_range():
    """Inside the range the error of a smooth input is uniform on [-step/2, step/2]: variance
    step^2/12 (the premise of the Irwin-Hall argument of Sec. 1)."""
    rng = np.random.default_rng(5)
    T, E = 4096, 64
    step = np.full((1, E), 2.0 ** -3, np.float32)
    _, inv = oracle.static_params(-step * 7.5, step * 7.5)
    x = rng.uniform(-0.9, 0.8, (T, E)).astype(np.float32)
    Y = f32_to_bf16_bits_lib(x)
    idx = np.zeros(0, np.int32)
    msg = oracle.encode_static(Y, idx, inv[0])
    xh = oracle.decode_reduce_static([msg], idx, step, oracle.ACC_FP32, out_fp32=True)
    err = (xh - bits_to_f32(Y)).astype(np.float64)
    assert np.abs(err).max() <= 2.0 ** -4
    var = err.var()
    assert abs(var / (2.0 ** -6 / 12) - 1) < 0.05
