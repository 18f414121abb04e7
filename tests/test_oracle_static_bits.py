"""Pins for the oracle's static symmetric mode at b-bit codes (Sec. 4 / Fig. 3: the paper varies
the bits of its own quantiser).  Reading: step = R / (2^b - 1), codes -2^(b-1) .. 2^(b-1) - 1,
field = code + 2^(b-1) in the row's little-endian bit string.

Checked against a hand-worked row, a float64 search over all levels, numpy's bit unpacking,
closed forms, numpy sums, and the separately written 4-bit routines.
"""
import numpy as np
import pytest

import oracle
from refmath import bits_to_f32, compaction, f32_to_bf16_bits_lib, f32_vals_to_bits

WIDTHS = (2, 3, 4, 5, 6, 8)


def unpack_bits(codes, r, b):
    bits = np.unpackbits(np.asarray(codes, np.uint8), axis=1, bitorder="little")
    body = bits[:, : r * b].reshape(codes.shape[0], r, b).astype(np.int64)
    return (body << np.arange(b)).sum(-1), bits[:, r * b:]


def test_worked_example_3_bits():
    """One device, 8 features, none selected, every feature calibrated to m = -3.5, M = 2:
    R = 2 * max(3.5, 2) = 7, step = 7 / 7 = 1, codes -4..3, field = code + 4.
    row   -5   -3.5  -2.5  -0.5  0.5  1.5  2.75  9
    x/1   -5   -3.5  -2.5  -0.5  0.5  1.5  2.75  9
    rint  -5   -4    -2    -0    0    2    3     9      (ties to even)
    clamp -4   -4    -2     0    0    2    3     3
    field  0    0     2     4    4    6    7     7
    bytes: 0 | 0<<3 | (2&3)<<6 = 0x80;  2>>2 | 4<<1 | 4<<4 | (6&1)<<7 = 0x48;  6>>1 | 7<<2 | 7<<5 = 0xFF"""
    E = 8
    idx = np.zeros(0, np.int32)
    m = np.full((1, E), -3.5, np.float32)
    M = np.full((1, E), 2.0, np.float32)
    step, inv = oracle.static_params(m, M, bits=3)
    assert step[0].tolist() == [1.0] * 8 and inv[0].tolist() == [1.0] * 8
    Y = f32_vals_to_bits(np.array([[-5, -3.5, -2.5, -0.5, 0.5, 1.5, 2.75, 9]], np.float32))
    msg = oracle.encode_static(Y, idx, inv[0], bits=3)
    assert msg.codes[0].tolist() == [0x80, 0x48, 0xFF]
    xh = oracle.decode_reduce_static([msg], idx, step, oracle.ACC_FP32, out_fp32=True, bits=3)
    assert xh[0].tolist() == [-4, -4, -2, 0, 0, 2, 3, 3]


@pytest.mark.parametrize("b", WIDTHS)
def test_params_closed_form(b):
    rng = np.random.default_rng(b)
    m = -np.abs(rng.standard_normal((2, 300))).astype(np.float32) * 10
    M = np.abs(rng.standard_normal((2, 300))).astype(np.float32) * 10
    m[0, :3] = [1.0, 0.0, -1e-31]
    M[0, :3] = [4.0, 0.0, 1e-31]
    step, inv = oracle.static_params(m, M, bits=b)
    qmax = np.float32(2 ** b - 1)
    R = (np.float32(2.0) * np.maximum(-m, M)).astype(np.float32)
    d = (R / qmax).astype(np.float32)
    live = d >= 1e-30
    assert np.array_equal(step, np.where(live, d, 0).astype(np.float32))
    with np.errstate(divide="ignore"):
        assert np.array_equal(inv, np.where(live, (np.float32(1.0) / d).astype(np.float32), 0).astype(np.float32))
    assert not live[0, 1] and not live[0, 2]


@pytest.mark.parametrize("b", WIDTHS)
@pytest.mark.parametrize("E,k,T", [(96, 0, 5), (104, 7, 4), (64, 64, 2), (40, 1, 6)])
def test_brute_force(E, k, T, b):
    """The chosen level is the nearest of the 2^b (float64 search); half a step inside the
    representable range, saturation outside; pad bits zero; selected features verbatim."""
    rng = np.random.default_rng(E * 100 + k * 10 + b)
    x = (rng.standard_normal((T, E)) * 3).astype(np.float32)
    Y = f32_to_bf16_bits_lib(x)
    xb = bits_to_f32(Y).astype(np.float64)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    m = np.full((1, E), -2.5, np.float32) * (1 + 0.1 * np.arange(E, dtype=np.float32) / E)
    M = np.full((1, E), 2.0, np.float32)
    m[0, ::9] = 0.0
    M[0, ::9] = 0.0                      # vanishing range: sent as 0
    step, inv = oracle.static_params(m, M, bits=b)
    msg = oracle.encode_static(Y, idx, inv[0], bits=b)
    r = E - k
    assert msg.codes.shape == (T, (r * b + 7) // 8)
    assert np.array_equal(msg.outl, Y[:, idx])
    if r == 0:
        return
    comp = compaction(idx, E)
    fields, pad = unpack_bits(msg.codes, r, b)
    assert not pad.any()
    half = 2 ** (b - 1)
    codes = fields - half
    assert codes.min() >= -half and codes.max() <= half - 1
    st = step[0, comp].astype(np.float64)
    xc = xb[:, comp]
    levels = np.arange(-half, half)[None, None, :] * st[None, :, None]
    dist = np.abs(xc[..., None] - levels)
    chosen = np.take_along_axis(dist, fields[..., None], -1)[..., 0]
    assert np.all(chosen <= dist.min(-1) + st * 2.0 ** -16 + np.abs(xc) * 2.0 ** -21)
    dead = st == 0
    assert np.all(codes[:, dead] == 0)
    inside = (xc >= -half * st) & (xc <= (half - 1) * st) & ~dead
    # (x * inv carries two fp32 roundings: up to |x| * 2^-22 beyond half a step)
    bound = 0.5 * st[None, :].repeat(T, 0) * (1 + 2.0 ** -18) + np.abs(xc) * 2.0 ** -22
    assert np.all(np.abs(codes * st - xc)[inside] <= bound[inside])
    assert np.all(codes[(xc > (half - 0.5) * st) & ~dead] == half - 1)
    assert np.all(codes[(xc < -(half + 0.5) * st) & ~dead] == -half)
    xh = oracle.decode_reduce_static([msg], idx, step, oracle.ACC_FP32, out_fp32=True, bits=b)
    assert np.array_equal(xh[:, comp], (codes.astype(np.float32) * step[0, comp]).astype(np.float32))
    assert np.array_equal(xh[:, idx], bits_to_f32(msg.outl))


def test_generic_routines_at_4_bits_equal_the_4_bit_routines():
    rng = np.random.default_rng(9)
    N, T, E, k = 3, 5, 136, 6
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    m = -np.abs(rng.standard_normal((N, E))).astype(np.float32) * 3
    M = np.abs(rng.standard_normal((N, E))).astype(np.float32) * 3
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 2) for _ in range(N)]
    s4, i4 = oracle.static_params(m, M)
    sg, ig = oracle.static_params(m, M, bits=4, generic=True)
    assert np.array_equal(s4, sg) and np.array_equal(i4, ig)
    a = [oracle.encode_static(Y, idx, i4[i]) for i, Y in enumerate(Ys)]
    g = [oracle.encode_static(Y, idx, i4[i], bits=4, generic=True) for i, Y in enumerate(Ys)]
    for x, y in zip(a, g):
        assert np.array_equal(x.codes, y.codes) and np.array_equal(x.outl, y.outl)
    for accum in (oracle.ACC_FP32, oracle.ACC_BF16):
        for out_fp32 in (False, True):
            assert np.array_equal(oracle.decode_reduce_static(a, idx, s4, accum, out_fp32),
                                  oracle.decode_reduce_static(a, idx, s4, accum, out_fp32, bits=4, generic=True))


@pytest.mark.parametrize("b", (2, 5, 8))
def test_decode_reduce_matches_numpy_rebuild(b):
    rng = np.random.default_rng(20 + b)
    N, T, E, k = 4, 6, 200, 8
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    comp = compaction(idx, E)
    m = -np.abs(rng.standard_normal((N, E))).astype(np.float32) * 3 - 1
    M = np.abs(rng.standard_normal((N, E))).astype(np.float32) * 3 + 1
    step, inv = oracle.static_params(m, M, bits=b)
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 2) for _ in range(N)]
    msgs = [oracle.encode_static(Y, idx, inv[i], bits=b) for i, Y in enumerate(Ys)]
    acc = None
    for i, mg in enumerate(msgs):
        fields, _ = unpack_bits(mg.codes, E - k, b)
        xh = np.empty((T, E), np.float32)
        xh[:, comp] = ((fields - 2 ** (b - 1)).astype(np.float32) * step[i, comp]).astype(np.float32)
        xh[:, idx] = bits_to_f32(mg.outl)
        acc = xh if acc is None else (acc + xh).astype(np.float32)
    assert np.array_equal(oracle.decode_reduce_static(msgs, idx, step, oracle.ACC_FP32, True, bits=b), acc)


@pytest.mark.parametrize("b", WIDTHS)
def test_bits_per_value_closed_form(b):
    """Nothing but codes and the BF16 features travels: b + (16 - b) k / E bits per value."""
    E, k, T = 5120, 80, 2
    Y = f32_to_bf16_bits_lib(np.random.default_rng(b).standard_normal((T, E)).astype(np.float32))
    idx = np.arange(0, E, 64, dtype=np.int32)
    inv = np.ones(E, np.float32)
    msg = oracle.encode_static(Y, idx, inv, bits=b)
    assert 8.0 * (msg.codes.shape[1] + 2 * msg.outl.shape[1]) / E == b + (16 - b) * k / E
