"""tpq_calibrate_fixed (the entry point that allocates nothing: its scratch is part of the
library's device image) against tpq_calibrate, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2411_07942_amd as tpq

pytestmark = pytest.mark.gpu


def _seq(S, E, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    y = torch.randn((S, E), generator=g) * 3.0
    y[:, ::97] *= 40.0
    return y.to(torch.bfloat16).cuda()


def _both(S, E, n_seq, seed):
    """(m, M) after n_seq sequences through tpq_calibrate and through tpq_calibrate_fixed."""
    N = 2
    m1 = torch.full((N, E), 5.0, device="cuda")
    M1 = torch.full((N, E), -5.0, device="cuda")
    m2, M2 = m1.clone(), M1.clone()
    ws = tpq.calibrate_workspace(S, E, "cuda")
    for s in range(n_seq):
        for rank in range(N):
            Y = _seq(S, E, seed + 10 * s + rank)
            tpq.calibrate(Y, rank, N, s, 0.25, m1, M1, ws)
            tpq.calibrate_fixed(Y, rank, N, s, 0.25, m2, M2)
    torch.cuda.synchronize()
    return m1.cpu().numpy(), M1.cpu().numpy(), m2.cpu().numpy(), M2.cpu().numpy()


def test_calibrate_fixed_matches_calibrate_two_calls_in_a_row():
    # a large call first, then a smaller one: the scratch keeps the first call's contents
    for S, E, n_seq in ((4096, 5120, 2), (200, 512, 3), (16384, 4608, 1), (7, 8, 2)):
        m1, M1, m2, M2 = _both(S, E, n_seq, seed=S + E)
        assert np.array_equal(m1.view(np.uint32), m2.view(np.uint32)), (S, E)
        assert np.array_equal(M1.view(np.uint32), M2.view(np.uint32)), (S, E)


def test_calibrate_fixed_rejects_what_does_not_fit():
    import ctypes
    lib = tpq._load()
    E = 8192 + 8
    Y = torch.zeros((8, E), dtype=torch.bfloat16, device="cuda")
    m = torch.zeros((1, E), device="cuda")
    M = torch.zeros((1, E), device="cuda")
    before = m.clone()
    rc = lib.tpq_calibrate_fixed(ctypes.c_void_p(Y.data_ptr()), 8, E, E, 0, 1, 0, ctypes.c_float(0.01),
                                 ctypes.c_void_p(m.data_ptr()), ctypes.c_void_p(M.data_ptr()), None)
    assert rc == tpq.ERR_SHAPE
    torch.cuda.synchronize()
    assert torch.equal(m, before)
