"""GPU parity of tpq_hop, the ring step (Sec. 5: the remark that the method could be adapted to
ring all-reduce): the outgoing message of every device is compared bit by bit with the oracle's
(decode the received message, add the device's partial sum, compress the bf16 result), in both
accumulation modes, including a whole ring of steps and the pad bytes of the outgoing buffers.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl
from gpu_common import CANARY, assert_message_equal, check_pad_bytes, gpu_encode, gpu_plan, idx_for

pytestmark = pytest.mark.gpu


def _ref(L, m, rows=None):
    outl, codes, scale, zero = m.to_dense(L)
    sel = (lambda a: a) if rows is None else (lambda a: a[rows])
    return oracle.Message(sel(outl), sel(codes), sel(scale), sel(zero))


def _case(E, G, Y_first, Y_own, idx, rows=None):
    """Devices i = 0 .. n-1 have received encode(Y_first[i]) and own Y_own[i]."""
    n = len(Y_first)
    T = Y_first[0].shape[0]
    L = tpq.layout_init(E, int(idx.size), G)
    plan = gpu_plan(L, idx)
    in_msgs = gpu_encode(L, plan, Y_first)
    sel = (lambda a: a) if rows is None else (lambda a: a[rows])
    for accum in (tpq.ACC_BF16, tpq.ACC_FP32):
        out_msgs = [tpq.Message(L, T, "cuda", fill=CANARY) for _ in range(n)]
        tpq.hop(L, plan, Y_own, in_msgs, out_msgs, accum)
        torch.cuda.synchronize()
        for i in range(n):
            want = oracle.hop(_ref(L, in_msgs[i], rows), sel(wl.to_bits(Y_own[i].contiguous())), idx, G, accum, threads=8)
            assert_message_equal(L, out_msgs[i], want, rows)
            check_pad_bytes(L, out_msgs[i], T)
    return L, plan


def _inputs(E, T, n, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    mk = lambda s: (torch.randn((T, E), generator=g, device="cuda") * s).to(torch.bfloat16)
    return [mk(1 + 5 * (i % 3)) for i in range(n)], [mk(2 + 3 * (i % 2)) for i in range(n)]


def test_tiny_config():
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    _case(w.E, w.G, Ys, Ys[1:] + Ys[:1], idx_for(w))


@pytest.mark.parametrize("E,k,G,T,n", [
    (512, 8, 128, 16, 4),
    (1032, 1, 128, 5, 3),      # odd r: a ragged last chunk
    (1027 * 8, 13, 64, 3, 2),  # ragged chunk, ragged group
    (1024, 0, 64, 7, 2),       # k = 0
    (64, 64, 32, 3, 2),        # k = E: only selected features
    (5120, 80, 128, 6, 8),     # Llama width
    (8192, 341, 64, 4, 16),    # the most devices one launch takes
    (2048, 600, 64, 5, 2),     # many selected features
    (8, 3, 32, 4, 2),
    (2048, 32, 32, 5, 3),
    (16384, 128, 256, 2, 1),   # widest group, two segments and more
])
def test_shapes_random_indices(E, k, G, T, n):
    first, own = _inputs(E, T, n, E + k)
    rng = np.random.default_rng(E + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    own[0][0] = 0           # a zero partial sum row
    first[-1][T - 1] = 0    # a received message of constant groups
    _case(E, G, first, own, idx)


def test_adjacent_selected_columns_and_row_stride():
    E, G, T = 1024, 128, 9
    idx = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, 100, 101, 511, 512, 1016, 1023], np.int32)
    first, own = _inputs(E, T, 2, 77)
    wide = [torch.zeros((T, E + 40), dtype=torch.bfloat16, device="cuda") for _ in own]
    for wd, y in zip(wide, own):
        wd[:, :E] = y
    _case(E, G, first, [wd[:, :E] for wd in wide], idx)


def test_a_ring_of_steps_matches_the_oracle_and_the_exact_sum():
    """encode on device 0, then N - 1 steps; the last message dequantised is close to the sum."""
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    idx = idx_for(w)
    L = tpq.layout_init(w.E, w.k, w.G)
    plan = gpu_plan(L, idx)
    msg = gpu_encode(L, plan, Ys[:1])[0]
    ref = oracle.encode(wl.to_bits(Ys[0]), idx, w.G)
    for y in Ys[1:]:
        nxt = tpq.Message(L, w.T, "cuda", fill=CANARY)
        tpq.hop(L, plan, [y], [msg], [nxt], tpq.ACC_BF16)
        torch.cuda.synchronize()
        ref = oracle.hop(ref, wl.to_bits(y), idx, w.G, oracle.ACC_BF16)
        assert_message_equal(L, nxt, ref)
        msg = nxt
    out = torch.empty((w.T, w.E), dtype=torch.float32, device="cuda")
    tpq.decode_reduce(L, plan, [msg], out, tpq.ACC_FP32)
    exact = sum(y.double() for y in Ys)
    steps = oracle.decode_reduce([ref], idx, w.E, w.G, oracle.ACC_FP32, out_fp32=True)
    assert np.array_equal(out.cpu().numpy(), steps)
    err = (out.double() - exact).abs()
    assert float(err.max()) <= 0.08 * float(exact.abs().max())


def test_llama_prefill_full_size():
    w = wl.LLAMA_PREFILL
    Ys = wl.partial_sums(w, device="cuda")
    _case(w.E, w.G, Ys, Ys[1:] + Ys[:1], idx_for(w))


def test_large_prefill_full_size():
    """16 devices side by side, [16384 x 8192], 4.5 bits (k = 341), group 64: sampled rows."""
    w = [v for v in wl.large_variants() if v.k == 341 and v.G == 64][0]
    Ys = wl.partial_sums(w, device="cuda")
    rng = np.random.default_rng(3)
    rows = np.unique(np.r_[0, 1, w.T - 1, rng.choice(w.T, 256, replace=False)])
    _case(w.E, w.G, Ys, Ys[3:] + Ys[:3], idx_for(w), rows=rows)
    del Ys
    torch.cuda.empty_cache()


def test_argument_errors():
    E, k, G = 512, 8, 128
    idx = np.arange(0, 24, 3).astype(np.int32)
    L = tpq.layout_init(E, k, G)
    L6 = tpq.layout_init(E, k, G, 6)
    plan = gpu_plan(L, idx)
    Y = [torch.zeros((2, E), dtype=torch.bfloat16, device="cuda")]
    a = [tpq.Message(L, 2, "cuda", fill=0)]
    b = [tpq.Message(L, 2, "cuda", fill=CANARY)]
    lib = tpq._load()
    p = lambda ms, name: tpq._ptr_array([getattr(m, name) for m in ms], 1)
    call = lambda Lx, n, accum: lib.tpq_hop(
        ctypes.byref(Lx), tpq._ptr(plan), tpq._ptr_array(Y, 1), E, n, 2,
        p(a, "codes"), p(a, "scale"), p(a, "zero"), p(a, "outl"), accum,
        p(b, "codes"), p(b, "scale"), p(b, "zero"), p(b, "outl"), None)
    assert call(L6, 1, tpq.ACC_BF16) == tpq.ERR_UNSUPPORTED
    assert call(L, 17, tpq.ACC_BF16) == tpq.ERR_SHAPE
    assert call(L, 1, 7) == tpq.ERR_UNSUPPORTED
    assert lib.tpq_hop(ctypes.byref(L), tpq._ptr(plan), tpq._ptr_array(Y, 1), E, 1, 2,
                       p(a, "codes"), p(a, "scale"), p(a, "zero"), None, tpq.ACC_BF16,
                       p(b, "codes"), p(b, "scale"), p(b, "zero"), p(b, "outl"), None) == tpq.ERR_NULL
    torch.cuda.synchronize()
    for t in (b[0].codes, b[0].scale, b[0].zero, b[0].outl):
        assert bool((t == CANARY).all().item()), "a refused call wrote to its outputs"
    assert call(L, 1, tpq.ACC_BF16) == 0
