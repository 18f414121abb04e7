"""Pins for the oracle's b-bit encode / decode_reduce (b in 2, 3, 4, 5, 6, 8: the
experiment of Sec. 4 / Fig. 3 that varies the number of bits of the quantised features).

Checked against definitions written independently of the oracle: a hand-worked example,
numpy's own bit unpacking, a float64 search over all 2^b levels, closed forms for the bit
count, numpy sums, the Irwin-Hall variance of summed errors (Sec. 1), and the separately
written 4-bit routines.
"""
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from refmath import (bits_to_f32, compaction, f32_to_bf16_bits_lib, f32_vals_to_bits,
                     group_expand)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bits_worked_example.txt")
WIDTHS = (2, 3, 4, 5, 6, 8)


def unpack_bits(codes, r, b):
    """[T,cb] bytes -> [T,r] codes and the pad bits, by numpy's little-endian bit order."""
    bits = np.unpackbits(np.asarray(codes, np.uint8), axis=1, bitorder="little")
    body = bits[:, : r * b].reshape(codes.shape[0], r, b).astype(np.int64)
    vals = (body << np.arange(b)).sum(-1)
    return vals, bits[:, r * b:]


def test_worked_example():
    spec = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            key, *rest = line.split()
            spec[key] = rest
    E, G = int(spec["E"][0]), int(spec["G"][0])
    idx = np.zeros(0, np.int32)
    Y = f32_vals_to_bits(np.array([[float(v) for v in spec["row"]]], np.float32))
    msg = oracle.encode(Y, idx, G, bits=3)
    assert msg.codes[0].tolist() == [int(v, 16) for v in spec["expect_codes"]]
    assert bits_to_f32(msg.scale)[0].tolist() == [float(v) for v in spec["expect_scale"]]
    assert bits_to_f32(msg.zero)[0].tolist() == [float(v) for v in spec["expect_zero"]]
    assert oracle.dequantize(msg, idx, E, G, bits=3)[0].tolist() == [float(v) for v in spec["expect_dequant"]]
    msg2 = oracle.encode(Y, idx, G, bits=2)
    assert msg2.codes[0].tolist() == [int(v, 16) for v in spec["bits2_expect_codes"]]
    assert bits_to_f32(msg2.scale)[0].tolist() == [float(v) for v in spec["bits2_expect_scale"]]
    assert oracle.dequantize(msg2, idx, E, G, bits=2)[0].tolist() == [float(v) for v in spec["bits2_expect_dequant"]]


def _check_against_definitions(Y, idx, G, b, msg):
    T, E = Y.shape
    k, r = idx.size, E - idx.size
    qmax = 2 ** b - 1
    assert msg.codes.shape == (T, (r * b + 7) // 8)          # closed form of the row length
    assert np.array_equal(msg.outl, Y[:, idx])               # selected features verbatim
    if r == 0:
        return
    comp = compaction(idx, E)
    xc = bits_to_f32(Y)[:, comp].astype(np.float64)
    ng = (r + G - 1) // G
    xp = np.pad(xc, ((0, 0), (0, ng * G - r)), mode="edge").reshape(T, ng, G)
    mn, mx = xp.min(2), xp.max(2)
    zero = bits_to_f32(msg.zero).astype(np.float64)
    assert np.array_equal(zero, mn + 0.0) and not np.any(msg.zero == 0x8000)
    s32 = ((mx - mn).astype(np.float32) / np.float32(qmax)).astype(np.float32)
    s_lib = f32_to_bf16_bits_lib(s32)
    degenerate = bits_to_f32(s_lib) < 1e-30
    assert np.array_equal(msg.scale, np.where(degenerate, 0, s_lib).astype(np.uint16))
    codes, pad = unpack_bits(msg.codes, r, b)
    assert not pad.any()
    assert codes.min() >= 0 and codes.max() <= qmax
    s_el = group_expand(bits_to_f32(msg.scale).astype(np.float64), G, r)
    z_el = group_expand(zero, G, r)
    levels = z_el[..., None] + np.arange(qmax + 1)[None, None, :] * s_el[..., None]
    dist = np.abs(xc[..., None] - levels)
    chosen = np.take_along_axis(dist, codes[..., None], -1)[..., 0]
    assert np.all(chosen <= dist.min(-1) + s_el * 2.0 ** -16)
    deg_el = group_expand(degenerate, G, r)
    assert np.all(codes[deg_el] == 0)
    # half a step, except where the bf16 rounding of the step pushes the top of the range
    # past the last level (at most qmax * 2^-8 steps, which exceeds half a step for b = 8)
    err = np.abs(z_el + codes * s_el - xc)
    slack = np.maximum(0.5, qmax * 2.0 ** -8 * (1 + 2.0 ** -12))
    assert np.all(err <= slack * s_el * (1 + 2.0 ** -18) + qmax * 1e-30)
    inner = codes < qmax
    assert np.all(err[inner] <= 0.5 * s_el[inner] * (1 + 2.0 ** -18) + qmax * 1e-30)
    is_max = xc == group_expand(mx, G, r)
    # the group maximum lands on the last level, unless rounding the step to bf16 (relative
    # 2^-8 at most) moves it by more than half a step: possible for b = 8 only
    top = codes[is_max & ~deg_el]
    assert np.all(top == qmax) if qmax * 2.0 ** -8 < 0.5 else np.all(top >= qmax - 1)
    assert np.all(err[xc == z_el] == 0)


@pytest.mark.parametrize("b", WIDTHS)
@pytest.mark.parametrize("E,k,G,T", [(96, 0, 32, 4), (104, 7, 32, 3), (520, 9, 128, 3),
                                     (64, 64, 32, 2), (40, 1, 8, 5), (16, 15, 4, 3)])
def test_brute_force_shapes(E, k, G, T, b):
    rng = np.random.default_rng(E * 1000 + k * 10 + b)
    x = rng.standard_normal((T, E)).astype(np.float32)
    x[:, ::7] *= 40
    x[0, :] = 0.0
    if T > 1:
        x[1, : E // 2] = -3.25
    Y = f32_to_bf16_bits_lib(x)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    msg = oracle.encode(Y, idx, G, bits=b)
    _check_against_definitions(Y, idx, G, b, msg)


def test_generic_routine_at_4_bits_equals_the_4_bit_routine():
    """Two separately written routines (nibble packing / bit-string packing) agree."""
    w = wl.TINY
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w)]
    cols, _ = wl.outlier_columns(w)
    idx = np.sort(cols.numpy()).astype(np.int32)
    a = [oracle.encode(Y, idx, w.G) for Y in Ys]
    g = [oracle.encode_bits(Y, idx, w.G, 4) for Y in Ys]
    for x, y in zip(a, g):
        assert np.array_equal(x.codes, y.codes) and np.array_equal(x.scale, y.scale)
        assert np.array_equal(x.zero, y.zero) and np.array_equal(x.outl, y.outl)
    for accum in (oracle.ACC_FP32, oracle.ACC_BF16):
        for out_fp32 in (False, True):
            assert np.array_equal(oracle.decode_reduce(a, idx, w.E, w.G, accum, out_fp32),
                                  oracle.decode_reduce(a, idx, w.E, w.G, accum, out_fp32, generic=True))


@pytest.mark.parametrize("b", WIDTHS)
def test_grid_inputs_round_trip_exactly(b):
    """Inputs on the code grid (every group spans 0..2^b - 1) come back bit for bit."""
    rng = np.random.default_rng(b)
    T, E, k, G = 6, 256, 4, 64
    qmax = 2 ** b - 1
    idx = np.array([3, 64, 65, 255], np.int32)
    comp = compaction(idx, E)
    q = rng.integers(0, qmax + 1, (T, E))
    for g0 in range(0, E - k, G):              # both ends of the range in every group
        q[:, comp[g0]] = 0
        q[:, comp[g0 + 1]] = qmax
    x = (q * 0.25 - 8.0).astype(np.float32)    # scale 0.25, zero -8: exact in bf16 for b <= 8
    Y = f32_vals_to_bits(x)
    msg = oracle.encode(Y, idx, G, bits=b)
    codes, _ = unpack_bits(msg.codes, E - k, b)
    assert np.array_equal(codes, q[:, comp])
    out = oracle.decode_reduce([msg], idx, E, G, oracle.ACC_FP32, out_fp32=False, bits=b)
    assert np.array_equal(out, Y)
    assert np.array_equal(oracle.decode_reduce([msg], idx, E, G, oracle.ACC_BF16, bits=b), Y)


@pytest.mark.parametrize("b", WIDTHS)
def test_decode_reduce_matches_numpy_rebuild(b):
    w = wl.TINY
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w)]
    cols, _ = wl.outlier_columns(w)
    idx = np.sort(cols.numpy()).astype(np.int32)
    msgs = [oracle.encode(Y, idx, w.G, bits=b) for Y in Ys]
    comp = compaction(idx, w.E)
    acc = None
    for mg in msgs:
        codes, _ = unpack_bits(mg.codes, w.r, b)
        s = group_expand(bits_to_f32(mg.scale), w.G, w.r)
        z = group_expand(bits_to_f32(mg.zero), w.G, w.r)
        xh = np.empty((w.T, w.E), np.float32)
        xh[:, comp] = (codes.astype(np.float32) * s + z).astype(np.float32)
        xh[:, idx] = bits_to_f32(mg.outl)
        acc = xh if acc is None else (acc + xh).astype(np.float32)
    out = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_FP32, out_fp32=True, bits=b)
    assert np.array_equal(out, acc)
    assert np.array_equal(oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_FP32, bits=b),
                          f32_to_bf16_bits_lib(acc))
    # the bf16 chain, exactly: every term and every partial sum through the library's conversion
    chain = None
    for mg in msgs:
        codes, _ = unpack_bits(mg.codes, w.r, b)
        s = group_expand(bits_to_f32(mg.scale), w.G, w.r)
        z = group_expand(bits_to_f32(mg.zero), w.G, w.r)
        xh = np.empty((w.T, w.E), np.float32)
        xh[:, comp] = (codes.astype(np.float32) * s + z).astype(np.float32)
        xh[:, idx] = bits_to_f32(mg.outl)
        term = bits_to_f32(f32_to_bf16_bits_lib(xh))
        chain = term if chain is None else bits_to_f32(f32_to_bf16_bits_lib((chain + term).astype(np.float32)))
    got = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_BF16, bits=b)
    assert np.array_equal(bits_to_f32(got), chain)


@pytest.mark.parametrize("b", (3, 6))
def test_summed_error_follows_irwin_hall(b):
    """Sec. 1: the error of N summed quantised values has variance N * step^2 / 12."""
    rng = np.random.default_rng(40 + b)
    N, T, E, G = 8, 64, 512, 128
    idx = np.zeros(0, np.int32)
    qmax = 2 ** b - 1
    msgs, exact = [], np.zeros((T, E), np.float64)
    for i in range(N):
        x = rng.uniform(-1.0, 1.0, (T, E)).astype(np.float32)
        x[:, ::G] = -1.0                      # every group spans exactly [-1, 1]
        x[:, 1::G] = 1.0
        Y = f32_to_bf16_bits_lib(x)
        exact += bits_to_f32(Y)
        msgs.append(oracle.encode(Y, idx, G, bits=b))
    step = float(bits_to_f32(msgs[0].scale)[0, 0])
    assert abs(step - 2.0 / qmax) <= 2.0 / qmax * 2.0 ** -8
    out = oracle.decode_reduce(msgs, idx, E, G, oracle.ACC_FP32, out_fp32=True, bits=b)
    err = (out.astype(np.float64) - exact).ravel()
    var = err.var()
    want = N * step * step / 12.0
    assert abs(var / want - 1.0) < 0.08, (var, want)


@pytest.mark.parametrize("b", WIDTHS)
def test_bits_per_value_closed_form(b):
    """b bits for the quantised features, 16 for the selected ones: b + (16 - b) k / E."""
    E, k, G, T = 5120, 80, 128, 2
    Y = f32_to_bf16_bits_lib(np.random.default_rng(b).standard_normal((T, E)).astype(np.float32))
    idx = np.arange(0, E, 64, dtype=np.int32)
    msg = oracle.encode(Y, idx, G, bits=b)
    payload = 8.0 * (msg.codes.shape[1] + 2 * msg.outl.shape[1]) / E
    assert payload == b + (16 - b) * k / E


def test_bad_width_is_refused():
    Y = np.zeros((1, 32), np.uint16)
    for b in (0, 1, 7, 9, 16):
        with pytest.raises(ValueError):
            oracle.encode(Y, np.zeros(0, np.int32), 32, bits=b)
