"""Pins for the oracle's calibration: Eq. (1), (2), R, Rbar, top-k (paper Sec. 3)."""
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from refmath import f32_vals_to_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ema_worked_example.txt")


def _parse_golden():
    devices, cur, seq = [], None, None
    top = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "gamma":
            top["gamma"] = float(rest[0])
        elif key == "E":
            top["E"] = int(rest[0])
        elif key == "device":
            cur = {"seqs": []}
            devices.append(cur)
        elif key == "seq":
            seq = []
            cur["seqs"].append(seq)
        elif key.startswith("expect_"):
            vals = [float(v) for v in rest]
            (cur if key in ("expect_m", "expect_M", "expect_R") else top)[key] = vals
        else:
            seq.append([float(v) for v in line.split()])
    return top, devices


def test_ema_worked_example_exact():
    top, devices = _parse_golden()
    E, N = top["E"], len(devices)
    m = np.zeros((N, E), np.float32)
    M = np.zeros((N, E), np.float32)
    for i, dev in enumerate(devices):
        for s, rows in enumerate(dev["seqs"]):
            Y = f32_vals_to_bits(np.array(rows, np.float32))
            oracle.calibrate_update(Y, m[i], M[i], first=(s == 0), gamma=top["gamma"])
        assert m[i].tolist() == dev["expect_m"]
        assert M[i].tolist() == dev["expect_M"]
    R, Rbar, idx_sorted, idx_ranked = oracle.calibrate_finalize(m, M, k=3)
    for i, dev in enumerate(devices):
        assert R[i].tolist() == dev["expect_R"]
    assert Rbar.tolist() == top["expect_Rbar"]
    assert idx_ranked.tolist() == [int(v) for v in top["expect_ranked"]]
    assert idx_sorted.tolist() == sorted(int(v) for v in top["expect_ranked"])
    # k = 1 and k = 2 take prefixes of the ranking
    for k in (1, 2):
        _, _, s_k, r_k = oracle.calibrate_finalize(m, M, k=k)
        assert r_k.tolist() == idx_ranked[:k].tolist()
        assert s_k.tolist() == sorted(idx_ranked[:k].tolist())


def _rand_bits(rng, S, E, scale=1.0):
    x = (rng.standard_normal((S, E)) * scale).astype(np.float32)
    return ((x.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)  # any bf16 values will do


def test_single_sequence_is_min_max():
    rng = np.random.default_rng(1)
    Y = _rand_bits(rng, 37, 24)
    m = np.full(24, 123.0, np.float32)
    M = np.full(24, -123.0, np.float32)
    oracle.calibrate_update(Y, m, M, first=True, gamma=0.01)
    v = wl.bits_to_f32(Y)
    assert np.array_equal(m, v.min(0)) and np.array_equal(M, v.max(0))


def test_gamma_one_keeps_only_last_sequence_and_constant_is_fixed_point():
    rng = np.random.default_rng(2)
    E = 16
    m = np.zeros(E, np.float32)
    M = np.zeros(E, np.float32)
    seqs = [_rand_bits(rng, 9, E) for _ in range(3)]
    for s, Y in enumerate(seqs):
        oracle.calibrate_update(Y, m, M, first=(s == 0), gamma=1.0)
    v = wl.bits_to_f32(seqs[-1])
    assert np.array_equal(m, v.min(0)) and np.array_equal(M, v.max(0))
    # the same sequence again and again: the state must stay where it is (up to
    # the rounding of (1-g)*m + g*m, which is within 1 ulp of m)
    m0, M0 = m.copy(), M.copy()
    for _ in range(50):
        oracle.calibrate_update(seqs[-1], m, M, first=False, gamma=0.01)
    assert np.allclose(m, m0, rtol=1e-5, atol=0) and np.allclose(M, M0, rtol=1e-5, atol=0)


def test_ema_matches_float64_recurrence():
    """gamma = 0.01 (the paper's constant): compare with the recurrence in float64."""
    rng = np.random.default_rng(3)
    E, n_seq = 64, 40
    m = np.zeros(E, np.float32)
    M = np.zeros(E, np.float32)
    m64 = M64 = None
    g = 0.01
    for s in range(n_seq):
        Y = _rand_bits(rng, 33, E, scale=1.0 + s % 5)
        oracle.calibrate_update(Y, m, M, first=(s == 0), gamma=g)
        v = wl.bits_to_f32(Y).astype(np.float64)
        if s == 0:
            m64, M64 = v.min(0), v.max(0)
        else:
            m64 = (1 - g) * m64 + g * v.min(0)
            M64 = (1 - g) * M64 + g * v.max(0)
    assert np.allclose(m, m64, rtol=2e-5, atol=1e-6)
    assert np.allclose(M, M64, rtol=2e-5, atol=1e-6)
    assert np.all(m <= M)


def test_zero_sign_is_canonical():
    # a column of mixed +0 / -0 must give +0 whichever comes first
    for first_bits in (0x0000, 0x8000):
        Y = np.array([[first_bits], [first_bits ^ 0x8000], [first_bits]], np.uint16)
        m = np.zeros(1, np.float32)
        M = np.zeros(1, np.float32)
        oracle.calibrate_update(Y, m, M, first=True)
        assert m.view(np.uint32)[0] == 0 and M.view(np.uint32)[0] == 0


def test_range_closed_form_and_topk_vs_numpy():
    rng = np.random.default_rng(4)
    N, E, k = 5, 300, 17
    m = -np.abs(rng.standard_normal((N, E))).astype(np.float32)
    M = np.abs(rng.standard_normal((N, E))).astype(np.float32)
    # some all-positive and all-negative columns, and exact ties
    m[:, :10] = np.abs(m[:, :10]) * 0.5
    M[:, :10] = np.abs(m[:, :10]) + 1
    M[:, 10:20] = -np.abs(M[:, 10:20]) * 0.5
    m[:, 10:20] = M[:, 10:20] - 1
    m[:, 100:140] = -2.0
    M[:, 100:140] = 1.0
    R, Rbar, idx_sorted, idx_ranked = oracle.calibrate_finalize(m, M, k)
    assert np.array_equal(R, 2 * np.maximum(-m, M))
    assert np.all(R >= 0)
    acc = R[0].copy()
    for i in range(1, N):
        acc = (acc + R[i]).astype(np.float32)
    assert np.array_equal(Rbar, acc)
    order = np.argsort(-Rbar.astype(np.float64), kind="stable")  # ties: lower index first
    assert idx_ranked.tolist() == order[:k].tolist()
    assert idx_sorted.tolist() == sorted(order[:k].tolist())
    # brute force: every selected feature's Rbar >= every unselected one's
    sel = np.zeros(E, bool)
    sel[idx_sorted] = True
    assert Rbar[sel].min() >= Rbar[~sel].max()


def test_ties_go_to_lower_index():
    N, E = 2, 12
    m = -np.ones((N, E), np.float32)
    M = np.ones((N, E), np.float32)
    _, _, idx_sorted, idx_ranked = oracle.calibrate_finalize(m, M, 4)
    assert idx_ranked.tolist() == [0, 1, 2, 3] and idx_sorted.tolist() == [0, 1, 2, 3]
    _, _, s0, _ = oracle.calibrate_finalize(m, M, 0)
    assert s0.size == 0


@pytest.mark.parametrize("w", [wl.TINY, wl.LLAMA_PREFILL])
def test_planted_outlier_columns_are_selected(w):
    """Columns planted with a range far above the base must all land in the top-k."""
    n_seq = min(4, wl.n_cal_sequences(w))
    m = np.zeros((w.N, w.E), np.float32)
    M = np.zeros((w.N, w.E), np.float32)
    for i in range(w.N):
        for s in range(n_seq):
            Y = wl.to_bits(wl.calibration_sequence(w, 0, i, s))
            oracle.calibrate_update(Y, m[i], M[i], first=(s == 0))
    _, _, idx_sorted, _ = oracle.calibrate_finalize(m, M, w.k)
    cols, _ = wl.outlier_columns(w, 0)
    assert set(cols.tolist()) <= set(idx_sorted.tolist())
    assert len(set(idx_sorted.tolist())) == w.k
