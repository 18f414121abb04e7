"""Seeded random shapes through every entry point of the hot path: for each seed one (E, k, G, T, N)
with a random set of selected features, a random run structure (isolated columns, adjacent
runs, columns at both ends of the row), rows of zeros and columns with outliers -- the dynamic
4-bit codec in all its modes, the static symmetric mode, one other code width, the fused
epilogue and the ring step, each compared bit by bit with the oracle by the helpers of the
per-feature test files."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2411_07942_amd as tpq
import workloads as wl
from test_gpu_bits import _case as bits_case
from test_gpu_fused import _case as fused_case
from test_gpu_hop import _case as hop_case
from test_gpu_parity import _codec_case
from test_gpu_static import _ranges_from, _static_case

pytestmark = pytest.mark.gpu


def _shape(seed):
    rng = np.random.default_rng(1000 + seed)
    E = 8 * int(rng.integers(1, 1300)) if seed % 6 else 8 * int(rng.integers(1300, 4097))
    G = int(rng.choice([32, 64, 128, 256]))
    kind = seed % 5
    if kind == 0:
        k = int(rng.integers(0, min(E, 9)))
    elif kind == 1:
        k = E // 64
    elif kind == 2:
        k = int(rng.integers(E // 16, E // 4 + 1))
    elif kind == 3:
        k = int(rng.integers(max(E - 40, 0), E + 1))
    else:
        k = int(rng.integers(0, E + 1))
    # selected features: some in adjacent runs, some at the ends, the rest anywhere
    chosen = set()
    if k and rng.random() < 0.5:
        chosen.add(0)
    if k > 1 and rng.random() < 0.5:
        chosen.add(E - 1)
    while len(chosen) < k:
        start = int(rng.integers(0, E))
        run = int(rng.integers(1, 12)) if rng.random() < 0.4 else 1
        for c in range(start, min(start + run, E)):
            if len(chosen) < k:
                chosen.add(c)
    idx = np.array(sorted(chosen), np.int32)
    T = int(rng.integers(1, 22))
    N = int(rng.integers(1, 10))
    return E, G, idx, T, N


def _data(E, T, N, idx, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(5000 + seed)
    Ys = []
    for i in range(N):
        x = torch.randn((T, E), generator=g, device="cuda") * (0.5 + i)
        if idx.size:
            x[:, torch.as_tensor(idx.astype(np.int64), device="cuda")] *= 30.0
        x[:, ::97] *= 12.0                     # outliers that were not selected
        if T > 2:
            x[T // 2] = 0.0                    # a row of zeros: every group constant
        Ys.append(x.to(torch.bfloat16))
    return Ys


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(seed):
    E, G, idx, T, N = _shape(seed)
    Ys = _data(E, T, N, idx, seed)
    w = dataclasses.replace(wl.TINY, N=N, T=T, E=E, k=int(idx.size), G=G)
    _codec_case(w, Ys, idx, ld_out=E + 8 * (seed % 3))
    m, M = _ranges_from(Ys)
    _static_case(E, G, Ys, idx, m, M)
    bits_case(E, G, (2, 3, 5, 6, 8)[seed % 5], Ys, idx)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    addend = (torch.randn((T, E), generator=g, device="cuda") * 3).to(torch.bfloat16)
    bias = (torch.randn((E,), generator=g, device="cuda") * 2).to(torch.bfloat16)
    fused_case(E, G, Ys, idx, addend if seed % 4 != 3 else None, bias if seed % 2 else None)
    own = _data(E, T, N, idx, seed + 100)
    hop_case(E, G, Ys, own, idx)


@pytest.mark.parametrize("E,G,cols,bits", [
    (5120, 128, [5 + 31 * i for i in range(80)], 3),
    (8192, 64, [3 + 11 * i for i in range(341)], 8),
    (8192, 128, [3 + 11 * i for i in range(300)] + list(range(3300, 3341)), 6),
], ids=["llama_width_first_segment", "large_width_two_segments", "large_width_with_run"])
def test_crowded_segments_in_every_mode(E, G, cols, bits):
    """Selected features crowded into part of the row, so that a segment has more cut chunks than
    the encoder's LDS area holds slots for: the static mode, another code width and the ring step
    run the same encoder code in kernels of their own."""
    T, N = 5, 2
    idx = np.array(sorted(set(cols)), np.int32)
    Ys = _data(E, T, N, idx, 900 + len(cols))
    m, M = _ranges_from(Ys)
    _static_case(E, G, Ys, idx, m, M)
    bits_case(E, G, bits, Ys, idx)
    hop_case(E, G, Ys, _data(E, T, N, idx, 901 + len(cols)), idx)
