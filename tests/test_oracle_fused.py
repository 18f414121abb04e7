"""Pins for the oracle's decode_reduce with the block's epilogue (Sec. 2: the output of a
row-parallel block is the sum over the devices plus the bias; an addend row -- a residual, or
the device's own partial sum when its message is left out -- enters the same way).

Checked against numpy / torch sums written independently of the oracle, closed forms on inputs
whose additions are exact, and the plain decode_reduce.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from refmath import bits_to_f32, compaction, f32_to_bf16_bits_lib, f32_vals_to_bits


def _tiny():
    w = wl.TINY
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w)]
    cols, _ = wl.outlier_columns(w)
    idx = np.sort(cols.numpy()).astype(np.int32)
    msgs = [oracle.encode(Y, idx, w.G) for Y in Ys]
    return w, Ys, idx, msgs


def test_without_epilogue_it_is_decode_reduce():
    w, Ys, idx, msgs = _tiny()
    for accum in (oracle.ACC_FP32, oracle.ACC_BF16):
        for out_fp32 in (False, True):
            a = oracle.decode_reduce(msgs, idx, w.E, w.G, accum, out_fp32)
            b = oracle.decode_reduce_fused(msgs, idx, w.E, w.G, None, None, accum, out_fp32)
            assert np.array_equal(a, b)


def test_epilogue_terms_follow_the_sum_fp32():
    """fp32 accumulate: out = ((sum) + addend) + bias, each one fp32 addition, one final rounding."""
    w, Ys, idx, msgs = _tiny()
    rng = np.random.default_rng(1)
    addend = f32_to_bf16_bits_lib(rng.standard_normal((w.T, w.E)).astype(np.float32) * 5)
    bias = f32_to_bf16_bits_lib(rng.standard_normal(w.E).astype(np.float32) * 3)
    base = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_FP32, out_fp32=True)
    want = (base + bits_to_f32(addend)).astype(np.float32)
    only_add = oracle.decode_reduce_fused(msgs, idx, w.E, w.G, addend, None, oracle.ACC_FP32, True)
    assert np.array_equal(only_add, want)
    want = (want + bits_to_f32(bias)[None, :]).astype(np.float32)
    both = oracle.decode_reduce_fused(msgs, idx, w.E, w.G, addend, bias, oracle.ACC_FP32, True)
    assert np.array_equal(both, want)
    assert np.array_equal(oracle.decode_reduce_fused(msgs, idx, w.E, w.G, addend, bias, oracle.ACC_FP32, False),
                          f32_to_bf16_bits_lib(want))
    only_bias = oracle.decode_reduce_fused(msgs, idx, w.E, w.G, None, bias, oracle.ACC_FP32, True)
    assert np.array_equal(only_bias, (base + bits_to_f32(bias)[None, :]).astype(np.float32))


def test_epilogue_terms_follow_the_sum_bf16_chain():
    """bf16 chain: each term is one more bf16 addition, as torch does it."""
    w, Ys, idx, msgs = _tiny()
    rng = np.random.default_rng(2)
    addend = f32_to_bf16_bits_lib(rng.standard_normal((w.T, w.E)).astype(np.float32) * 5)
    bias = f32_to_bf16_bits_lib(rng.standard_normal(w.E).astype(np.float32) * 3)
    base = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_BF16, out_fp32=False)
    t = wl.from_bits(base) + wl.from_bits(addend)
    t = t + wl.from_bits(bias)[None, :]
    got = oracle.decode_reduce_fused(msgs, idx, w.E, w.G, addend, bias, oracle.ACC_BF16, False)
    assert np.array_equal(got, wl.to_bits(t))


def test_distinct_bias_per_column_lands_on_its_column():
    """Exact arithmetic (small multiples of 1/4): out - plain = addend + bias, column by column,
    selected columns included."""
    rng = np.random.default_rng(3)
    N, T, E, k, G = 3, 4, 128, 5, 32
    idx = np.array([0, 17, 64, 65, 127], np.int32)
    comp = compaction(idx, E)
    Ys = []
    for i in range(N):
        q = rng.integers(0, 16, (T, E))
        for g0 in range(0, E - k, G):
            q[:, comp[g0]] = 0
            q[:, comp[g0 + 1]] = 15
        Ys.append(f32_vals_to_bits((q * 0.25 - 2.0).astype(np.float32)))
    msgs = [oracle.encode(Y, idx, G) for Y in Ys]
    bias = f32_vals_to_bits((np.arange(E) * 0.25).astype(np.float32))                 # distinct per column
    addend = f32_vals_to_bits((np.arange(T)[:, None] * 4.0 + (np.arange(E)[None, :] % 8) * 0.5).astype(np.float32))
    plain = oracle.decode_reduce(msgs, idx, E, G, oracle.ACC_FP32, out_fp32=True)
    got = oracle.decode_reduce_fused(msgs, idx, E, G, addend, bias, oracle.ACC_FP32, True)
    assert np.array_equal(got - plain, bits_to_f32(addend) + bits_to_f32(bias)[None, :])
    exact = sum(bits_to_f32(Y).astype(np.float64) for Y in Ys)
    assert np.array_equal(got.astype(np.float64), exact + bits_to_f32(addend) + bits_to_f32(bias)[None, :])


def test_k_equals_E_is_the_textbook_block_output():
    """Everything in BF16: sum of the devices' tensors + residual + bias."""
    rng = np.random.default_rng(4)
    N, T, E = 4, 6, 48
    idx = np.arange(E, dtype=np.int32)
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 3) for _ in range(N)]
    res = f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32))
    bias = f32_to_bf16_bits_lib(rng.standard_normal(E).astype(np.float32))
    msgs = [oracle.encode(Y, idx, 32) for Y in Ys]
    acc = bits_to_f32(Ys[0]).copy()
    for Y in Ys[1:]:
        acc = (acc + bits_to_f32(Y)).astype(np.float32)
    acc = (acc + bits_to_f32(res)).astype(np.float32)
    acc = (acc + bits_to_f32(bias)[None, :]).astype(np.float32)
    assert np.array_equal(oracle.decode_reduce_fused(msgs, idx, E, 32, res, bias, oracle.ACC_FP32, True), acc)
    t = wl.from_bits(Ys[0]).clone()
    for Y in Ys[1:]:
        t = t + wl.from_bits(Y)
    t = (t + wl.from_bits(res)) + wl.from_bits(bias)[None, :]
    assert np.array_equal(oracle.decode_reduce_fused(msgs, idx, E, 32, res, bias, oracle.ACC_BF16, False),
                          wl.to_bits(t))


def test_own_partial_sum_unquantised():
    """A device leaves its own message out and adds its exact partial sum instead: with one other
    device, out = dequantised other + own, and with no quantisation error on the own part."""
    w, Ys, idx, msgs = _tiny()
    other = oracle.dequantize(msgs[0], idx, w.E, w.G)
    got = oracle.decode_reduce_fused([msgs[0]], idx, w.E, w.G, Ys[1], None, oracle.ACC_FP32, True)
    assert np.array_equal(got, (other + bits_to_f32(Ys[1])).astype(np.float32))
    # the error against the exact sum is the other device's quantisation error alone
    exact = bits_to_f32(Ys[0]).astype(np.float64) + bits_to_f32(Ys[1])
    err_own_exact = np.abs(got - exact)
    both_q = oracle.decode_reduce(msgs[:2], idx, w.E, w.G, oracle.ACC_FP32, out_fp32=True)
    assert err_own_exact.mean() < np.abs(both_q - exact).mean()
