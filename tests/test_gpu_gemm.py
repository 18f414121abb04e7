"""GPU parity of the linear layer with the compression in its epilogue (tpq_gemm_weights,
tpq_gemm_encode; Sec. 2: f^(i)(x^(i)) = x^(i) W^(i) is what C^(i) compresses).

Three bars.  (1) The rounded product the kernel keeps (Y_msg) against the oracle's linear layer
(float64 sum, one rounding): the matrix cores add the K products in an order of their own, in
fp32, so the bar is one bf16 ulp plus the fp32 accumulation bound K * 2^-24 * sum |x w|, with the
share of bit-identical values reported; on small-integer inputs every sum is exact and the
product must be identical.  (2) Given that product, the message must be the oracle's encode of
it, bit for bit.  (3) End to end against oracle.encode(oracle.linear(...)): identical on exact
inputs; on general inputs the selected features within one ulp, and codes within one step
wherever the group's scale and zero agree.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl
from gpu_common import CANARY, assert_message_equal, bits_to_f32, check_pad_bytes, gpu_plan

pytestmark = pytest.mark.gpu


def _order(E, idx):
    """Message order: the features that are quantised, ascending, then the selected ones."""
    rest = np.setdiff1d(np.arange(E), idx)
    return np.concatenate([rest, idx]).astype(np.int64)


def _ulp_bf16(x):
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -126))) - 7)


def _run(T, K, E, k, G, seed, integer=False, ld_pad=0, rows=None, want_y=True, idx=None):
    rng = np.random.default_rng(seed)
    if idx is None:
        idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    X, Wt = wl.linear_inputs(T, K, E, idx, seed, device="cuda", integer=integer)
    if ld_pad:
        Xb = torch.zeros((T, K + ld_pad), dtype=torch.bfloat16, device="cuda")
        Xb[:, :K] = X
        X = Xb[:, :K]
    L = tpq.layout_init(E, k, G)
    plan = gpu_plan(L, idx)
    Wp = tpq.gemm_weights(L, plan, Wt)
    order = _order(E, idx)
    assert torch.equal(Wp, Wt[torch.as_tensor(order, device="cuda")]), "weights are not in message order"

    msg = tpq.Message(L, T, "cuda", fill=CANARY)
    Ybuf = torch.full((T, E + 8), 777.0, dtype=torch.bfloat16, device="cuda")
    tpq.gemm_encode(L, X, Wp, msg, Ybuf[:, :E] if want_y else None)
    torch.cuda.synchronize()
    check_pad_bytes(L, msg, T)
    if not want_y:
        return L, idx, msg, None
    assert bool((Ybuf[:, E:] == 777.0).all().item()), "wrote past the product's rows"
    Ym = wl.to_bits(Ybuf[:, :E].contiguous())
    Yg = np.empty_like(Ym)
    Yg[:, order] = Ym                       # back to original feature order (format conversion only)

    sel = np.arange(T) if rows is None else np.asarray(rows)
    # (2) given the product, the message is the oracle's encode of it
    ref = oracle.encode(Yg[sel], idx, G, threads=8)
    assert_message_equal(L, msg, ref, None if rows is None else sel)

    # (1) the product
    Xs = wl.to_bits(X.contiguous())[sel]
    Yo, mag = oracle.linear(Xs, wl.to_bits(Wt), threads=8, with_magnitude=True)
    g, o = bits_to_f32(Yg[sel]).astype(np.float64), bits_to_f32(Yo).astype(np.float64)
    same = float(np.mean(Yg[sel] == Yo))
    if integer:
        assert np.array_equal(Yg[sel], Yo), "exact inputs: the product must be identical"
    else:
        bound = _ulp_bf16(np.maximum(np.abs(g), np.abs(o))) + 2.0 * K * 2.0 ** -24 * mag
        assert np.all(np.abs(g - o) <= bound), float(np.max(np.abs(g - o) / bound))
        assert same >= 0.97, same
    # (3) end to end
    ref2 = oracle.encode(Yo, idx, G, threads=8)
    outl, codes, scale, zero = (a if rows is None else a[sel] for a in msg.to_dense(L))
    if integer:
        assert_message_equal(L, msg, ref2, None if rows is None else sel)
    else:
        if k:
            a, b = bits_to_f32(outl).astype(np.float64), bits_to_f32(ref2.outl).astype(np.float64)
            mo = mag[:, idx]
            assert np.all(np.abs(a - b) <= _ulp_bf16(np.maximum(np.abs(a), np.abs(b))) + 2.0 * K * 2.0 ** -24 * mo)
        if L.r:
            agree = (scale == ref2.scale) & (zero == ref2.zero)          # [rows, ng]
            r = L.r
            lo = (codes & 0x0F).astype(np.int16)
            hi = (codes >> 4).astype(np.int16)
            cg = np.stack([lo, hi], axis=2).reshape(codes.shape[0], -1)[:, :r]
            lo2 = (ref2.codes & 0x0F).astype(np.int16)
            hi2 = (ref2.codes >> 4).astype(np.int16)
            co = np.stack([lo2, hi2], axis=2).reshape(codes.shape[0], -1)[:, :r]
            grp = np.arange(r) // G
            ok_grp = agree[:, grp]
            assert np.all(np.abs(cg - co)[ok_grp] <= 1), "codes more than one step apart"
            assert agree.mean() >= 0.9, agree.mean()
    return L, idx, msg, same


@pytest.mark.parametrize("T,K,E,k,G", [
    (200, 96, 512, 8, 128),       # two feature tiles, two token tiles, ragged T
    (70, 1728, 5120, 80, 128),    # Llama width and depth of one device's slice
    (130, 40, 264, 5, 32),        # K and E off the tile sizes, groups of 32
    (64, 64, 1024, 16, 64),       # groups of 64
    (129, 128, 1024, 16, 256),    # groups of 256: two waves share a group
    (5, 32, 1032, 1, 128),        # odd r: a pad nibble
    (33, 64, 768, 0, 128),        # k = 0
    (17, 64, 256, 256, 32),       # k = E: everything stays bf16
    (1, 8, 64, 3, 32),            # one token, one piece of k
    (300, 512, 4608, 72, 128),    # Gemma width
    (40, 64, 8192, 341, 64),      # odd r = 7851, the outlier section spans two tiles
])
def test_general_inputs(T, K, E, k, G):
    _run(T, K, E, k, G, seed=T + K + E)


@pytest.mark.parametrize("T,K,E,k,G", [
    (200, 96, 512, 8, 128),
    (130, 40, 264, 5, 32),
    (129, 128, 1024, 16, 256),
    (64, 160, 1024, 16, 64),
])
def test_exact_inputs_are_bit_exact_end_to_end(T, K, E, k, G):
    _run(T, K, E, k, G, seed=3 * T + K, integer=True)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(seed):
    """Seeded random (E, k, G) with selected features in runs and at both ends of the row (the
    generator of test_gpu_random_shapes), random T and K."""
    from test_gpu_random_shapes import _shape
    E, G, idx, _, _ = _shape(seed)
    rng = np.random.default_rng(77 + seed)
    T = int(rng.integers(1, 300))
    K = 8 * int(rng.integers(1, 66))
    _run(T, K, E, int(idx.size), G, seed=seed, integer=bool(seed % 4 == 3), idx=idx)


def test_padded_rows_and_no_product_output():
    L, idx, msg_a, _ = _run(77, 96, 512, 8, 128, seed=5, ld_pad=24)
    L, idx, msg_b, _ = _run(77, 96, 512, 8, 128, seed=5, ld_pad=24, want_y=False)
    for a, b in zip(msg_a.to_dense(L), msg_b.to_dense(L)):
        assert np.array_equal(a, b)


def test_llama_shape_full_size_sampled_rows():
    """One device's real call at the Llama-2-13B shape (down projection: K = 13824 / 8): every row
    is produced, the message is checked on every row, the product on a sample of rows."""
    T, K, E, k, G = 2048, 1728, 5120, 80, 128
    rows = np.unique(np.concatenate([np.arange(0, T, 37), [T - 1]]))
    _run(T, K, E, k, G, seed=11, rows=rows)


def test_argument_errors():
    L = tpq.layout_init(512, 8, 128)
    X = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    Wp = torch.zeros((512, 64), dtype=torch.bfloat16, device="cuda")
    msg = tpq.Message(L, 4, "cuda")
    lib = tpq._load()
    import ctypes
    def call(K, ldX):
        return lib.tpq_gemm_encode(ctypes.byref(L), X.data_ptr(), 4, ldX, K, Wp.data_ptr(), msg.codes.data_ptr(),
                                   msg.scale.data_ptr(), msg.zero.data_ptr(), msg.outl.data_ptr(), None, 0, None)
    assert call(64, 64) == 0
    assert call(60, 64) != 0      # K not a multiple of 8
    assert call(64, 56) != 0      # row stride below K
    assert call(0, 64) != 0
    L8 = tpq.layout_init(512, 8, 128, bits=8)
    assert lib.tpq_gemm_encode(ctypes.byref(L8), X.data_ptr(), 4, 64, 64, Wp.data_ptr(), msg.codes.data_ptr(),
                               msg.scale.data_ptr(), msg.zero.data_ptr(), msg.outl.data_ptr(), None, 0, None) != 0
    torch.cuda.synchronize()
