"""Pins for the oracle's ring step (Sec. 5: the remark that the method could be adapted to ring
all-reduce; the reading taken here: a device dequantises the message it receives, adds its own
bf16 partial sum as one more term of the accumulation, and compresses the bf16 result again).

Checked against the same steps written with numpy / torch in this file (nothing of the oracle
but the message under test), the encoder's definitional checks on the result, a closed form
(values on an exactly representable grid come back unchanged), and the error bound of a whole
ring of steps.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from refmath import bits_to_f32, compaction, f32_to_bf16_bits_lib, f32_vals_to_bits, group_expand, unpack_codes
from test_oracle_codec import _check_message_against_definitions


def _bf16_add(a_bits, b_bits):
    """a + b as torch adds two bf16 tensors."""
    ta = torch.from_numpy(np.ascontiguousarray(a_bits).view(np.int16)).view(torch.bfloat16)
    tb = torch.from_numpy(np.ascontiguousarray(b_bits).view(np.int16)).view(torch.bfloat16)
    return (ta + tb).view(torch.int16).numpy().view(np.uint16)


def _independent_sum(msg, Y, idx, G, accum):
    """bf16 bits [T,E] of (dequantised message) (+) Y, written without the oracle."""
    T, E = Y.shape
    comp = compaction(idx, E)
    r = comp.size
    out = np.empty((T, E), np.uint16)
    if idx.size:
        out[:, idx] = _bf16_add(msg.outl, Y[:, idx])
    if r:
        codes, _ = unpack_codes(msg.codes, r)
        s = group_expand(bits_to_f32(msg.scale), G, r)
        z = group_expand(bits_to_f32(msg.zero), G, r)
        xh = (codes.astype(np.float32) * s + z).astype(np.float32)   # the product is exact
        if accum == oracle.ACC_BF16:
            out[:, comp] = _bf16_add(f32_to_bf16_bits_lib(xh), Y[:, comp])
        else:
            out[:, comp] = f32_to_bf16_bits_lib((xh + bits_to_f32(Y[:, comp])).astype(np.float32))
    return out


def _same(a, b):
    return (np.array_equal(a.outl, b.outl) and np.array_equal(a.codes, b.codes) and
            np.array_equal(a.scale, b.scale) and np.array_equal(a.zero, b.zero))


@pytest.mark.parametrize("accum", [oracle.ACC_BF16, oracle.ACC_FP32])
def test_tiny_config_against_the_steps_written_out(accum):
    w = wl.TINY
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w)]
    cols, _ = wl.outlier_columns(w)
    idx = np.sort(cols.numpy()).astype(np.int32)
    msg = oracle.encode(Ys[0], idx, w.G)
    for Y in Ys[1:]:
        nxt = oracle.hop(msg, Y, idx, w.G, accum)
        V = _independent_sum(msg, Y, idx, w.G, accum)
        _check_message_against_definitions(V, idx, w.G, nxt)
        assert _same(nxt, oracle.encode(V, idx, w.G))
        msg = nxt


@pytest.mark.parametrize("E,k,G,T", [(96, 0, 32, 5), (104, 7, 32, 3), (256, 11, 64, 6), (520, 9, 128, 3),
                                     (64, 64, 32, 2), (40, 1, 8, 9)])
@pytest.mark.parametrize("accum", [oracle.ACC_BF16, oracle.ACC_FP32])
def test_shapes_against_the_steps_written_out(E, k, G, T, accum):
    """ragged last group, odd r, k = 0, k = E"""
    rng = np.random.default_rng(E * 100 + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    Y0 = f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 3)
    Y1 = f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 3)
    Y1[0] = 0
    msg = oracle.encode(Y0, idx, G)
    nxt = oracle.hop(msg, Y1, idx, G, accum)
    V = _independent_sum(msg, Y1, idx, G, accum)
    _check_message_against_definitions(V, idx, G, nxt)
    assert _same(nxt, oracle.encode(V, idx, G))


def test_grid_values_come_back_unchanged():
    """A group whose values are zero + q * 2^e with codes 0 and 15 present is represented exactly;
    adding a zero partial sum and compressing again must give the same message."""
    E, G, T = 256, 64, 4
    rng = np.random.default_rng(5)
    idx = np.array([3, 100, 101], np.int32)
    q = rng.integers(0, 16, (T, E)).astype(np.float32)
    q[:, ::16] = 0
    q[:, 1::16] = 15
    x = (q * np.float32(0.25) - np.float32(2.0)).astype(np.float32)   # 8-bit significands: bf16 values
    Y0 = f32_vals_to_bits(x)
    msg = oracle.encode(Y0, idx, G)
    assert np.array_equal(oracle.decode_reduce([msg], idx, E, G, oracle.ACC_BF16), Y0)
    for accum in (oracle.ACC_BF16, oracle.ACC_FP32):
        assert _same(oracle.hop(msg, np.zeros((T, E), np.uint16), idx, G, accum), msg)


def test_selected_features_are_added_in_bf16():
    E, G, T = 64, 32, 2
    idx = np.array([5, 40], np.int32)
    Y0 = f32_vals_to_bits(np.full((T, E), 1.0, np.float32))
    Y1 = f32_vals_to_bits(np.full((T, E), 2.0 ** -8, np.float32))      # half an ulp of 1.0 in bf16
    Y0[:, 5] = f32_vals_to_bits(np.float32(1.0078125))                  # 1 + 2^-7: odd last bit
    nxt = oracle.hop(oracle.encode(Y0, idx, G), Y1, idx, G)
    # 1 + 2^-8 is a tie and goes to the even neighbour 1; 1 + 2^-7 + 2^-8 goes up to 1 + 2^-6
    assert np.array_equal(bits_to_f32(nxt.outl[:, 1]), np.full(T, 1.0, np.float32))
    assert np.array_equal(bits_to_f32(nxt.outl[:, 0]), np.full(T, 1.015625, np.float32))


@pytest.mark.parametrize("N", [2, 4, 8])
def test_a_ring_of_steps_stays_within_the_sum_of_half_steps(N):
    """encode, then N - 1 ring steps: every step adds at most half its own quantisation step and
    the bf16 roundings of the running sum."""
    T, E, G = 8, 512, 128
    rng = np.random.default_rng(N)
    idx = np.sort(rng.choice(E, 8, replace=False)).astype(np.int32)
    comp = compaction(idx, E)
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32)) for _ in range(N)]
    msg = oracle.encode(Ys[0], idx, G)
    bound = 0.5 * group_expand(bits_to_f32(msg.scale).astype(np.float64), G, comp.size)
    exact = bits_to_f32(Ys[0]).astype(np.float64)
    for Y in Ys[1:]:
        msg = oracle.hop(msg, Y, idx, G, oracle.ACC_BF16)
        exact = exact + bits_to_f32(Y).astype(np.float64)
        # two bf16 roundings of a value below 2 * max|sum| per step, then half the new step
        bound = bound + 2 * 2.0 ** -8 * (np.abs(exact[:, comp]) + bound) + \
            0.5 * group_expand(bits_to_f32(msg.scale).astype(np.float64), G, comp.size) * (1 + 2.0 ** -7)
    got = oracle.decode_reduce([msg], idx, E, G, oracle.ACC_FP32, out_fp32=True).astype(np.float64)
    assert np.all(np.abs(got[:, comp] - exact[:, comp]) <= bound)
    # selected features: bf16 additions only
    assert np.all(np.abs(got[:, idx] - exact[:, idx]) <= N * 2.0 ** -8 * (np.abs(exact[:, idx]) + 1))
