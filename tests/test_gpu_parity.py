"""GPU parity: the HIP library against the CPU oracle on the same seeded inputs.

Bars: packed codes, scales, zeros, outlier values and indices bit-exact; reduced
sums within 1e-5 (fp32 accumulate) / 1e-2 (bf16 accumulate) of the summation's
natural scale -- and, where the GPU evaluates in the oracle's order, bit-exact.
All calls go through the C ABI (ctypes binding).
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl
from gpu_common import (bits_to_f32, CANARY, assert_message_equal, check_pad_bytes, gpu_decode, gpu_encode,
                        gpu_plan, idx_for, sum_tolerance_fraction, sum_tolerance_ok)
from refmath import compaction

pytestmark = pytest.mark.gpu


def _codec_case(w, Ys_dev, idx, rows=None, modes=((tpq.ACC_FP32, False), (tpq.ACC_FP32, True),
                                                   (tpq.ACC_BF16, False), (tpq.ACC_FAST, False)), ld_out=None):
    """Encode + decode on the GPU, oracle on (a sample of) the rows, compare."""
    L = tpq.layout_init(w.E, idx.size, w.G)
    plan = gpu_plan(L, idx)
    T = Ys_dev[0].shape[0]
    msgs = gpu_encode(L, plan, Ys_dev)
    sel = slice(None) if rows is None else rows
    refs = []
    for i, y in enumerate(Ys_dev):
        Y = wl.to_bits(y[sel] if rows is None else y[torch.as_tensor(rows, device=y.device)])
        ref = oracle.encode(Y, idx, w.G, threads=8)
        assert_message_equal(L, msgs[i], ref, rows)
        check_pad_bytes(L, msgs[i], T)
        refs.append(ref)
    for accum, out_fp32 in modes:
        got, guard_ok = gpu_decode(L, plan, msgs, T, accum, out_fp32, ld=ld_out)
        assert guard_ok, "decode wrote outside its rows"
        if rows is not None:
            got = got[rows]
        if accum == tpq.ACC_FAST:
            # The bf16 mode at its tolerance.  Against the oracle's literal bf16 chain: every
            # element within the chain's own rounding bound, (N + 1) * 2^-9 * sum |x_hat_i| (N
            # roundings of terms and partial sums at 2^-9 each, the fp32 sum being exact to
            # 2^-20), and all but a few per million within the 1e-2 bar itself (the exceptions
            # are where the chain's accumulated rounding exceeds 1e-2, not where this mode errs:
            # against the exact sum it stays within half a bf16 ulp) ...
            chain = oracle.decode_reduce(refs, idx, w.E, w.G, tpq.ACC_BF16, out_fp32=out_fp32, threads=8)
            n_terms = len(refs)
            assert sum_tolerance_ok(got, chain, refs, idx, w.E, w.G, out_fp32, (n_terms + 1) * 2.0 ** -9)
            frac, _ = sum_tolerance_fraction(got, chain, refs, idx, w.E, w.G, out_fp32, 1e-2)
            assert frac >= 0.9995, frac
            # ... and evaluated as the fp32 chain, so identical to that
            want = oracle.decode_reduce(refs, idx, w.E, w.G, tpq.ACC_FP32, out_fp32=out_fp32, threads=8)
            assert np.array_equal(got, want), "fast mode differs from the fp32 chain"
            # ... which puts it within half a bf16 ulp (one rounding) of the exact sum of the dequantised
            # messages, up to the fp32 additions' own rounding (n_terms * 2^-24 of the magnitudes)
            exact = np.zeros(got.shape, np.float64)
            mag = np.zeros(got.shape, np.float64)
            for mg in refs:
                x = oracle.dequantize(mg, idx, w.E, w.G).astype(np.float64)
                exact += x
                mag += np.abs(x)
            g64 = (got if out_fp32 else bits_to_f32(got)).astype(np.float64)
            half_ulp = 0.0 if out_fp32 else 2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 2.0 ** -126))) - 8)
            assert np.all(np.abs(g64 - exact) <= half_ulp * (1 + 2.0 ** -7) + n_terms * 2.0 ** -24 * mag + 1e-37)
            continue
        want = oracle.decode_reduce(refs, idx, w.E, w.G, accum, out_fp32=out_fp32, threads=8)
        rel = 1e-2 if accum == tpq.ACC_BF16 else 1e-5
        assert sum_tolerance_ok(got, want, refs, idx, w.E, w.G, out_fp32, rel)
        # the kernels follow the oracle's evaluation order, so the sums are identical too
        assert np.array_equal(got, want), "sums within tolerance but not bit-identical"
    return L, msgs


def test_tiny_config_all_modes():
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    _codec_case(w, Ys, idx_for(w))


@pytest.mark.parametrize("E,k,G,T,N", [
    (512, 8, 128, 16, 4),      # ragged last group (120)
    (1032, 1, 128, 5, 3),      # odd r: pad nibble; T not a multiple of anything
    (1024, 0, 64, 7, 2),       # k = 0: the plain Int4 baseline
    (64, 64, 32, 3, 2),        # k = E: everything in bf16
    (96, 95, 32, 4, 2),        # a single quantised feature
    (4608, 72, 128, 9, 8),     # Gemma width: 36 groups, last of 56
    (5120, 80, 128, 6, 8),     # Llama width: 40 groups, last of 48
    (8192, 341, 64, 4, 16),    # odd r = 7851, 123 groups, last of 43
    (8192, 128, 256, 3, 2),    # 32 lanes per group
    (2048, 32, 32, 5, 5),      # 4 lanes per group
    (520, 9, 128, 1, 1),       # one row, one rank
    (2048, 600, 64, 5, 2),     # many selected features: the encoder's whole-row LDS path
    (4096, 497, 128, 3, 2),    # just past the streaming path's limit on k
    (4096, 496, 128, 3, 2),    # ... and just inside it
    (32768, 512, 128, 2, 2),   # the widest row the library takes
    (8, 3, 32, 4, 2),          # the narrowest
])
def test_shapes_random_indices(E, k, G, T, N):
    """Random selected features (the paper's "Random BF16" baseline is this case)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(E * 31 + k)
    Ys = []
    for i in range(N):
        x = torch.randn((T, E), generator=g, device="cuda")
        x[:, ::11] *= 37.0
        x[0, : E // 2] = 0.0                       # constant (degenerate) groups
        if T > 1:
            x[1] = -1.5
        if T > 2:
            x[2, ::2] = 0.0
            x[2, 1::2] = -0.0
        Ys.append(x.to(torch.bfloat16))
    rng = np.random.default_rng(E + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    w = dataclasses.replace(wl.TINY, N=N, T=T, E=E, k=k, G=G)
    _codec_case(w, Ys, idx, ld_out=E + 16)


def test_adjacent_and_edge_outliers():
    """Selected features in runs, at column 0 and at column E-1."""
    E, G, T, N = 1024, 128, 4, 3
    idx = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, 100, 101, 511, 512, 513, 1015, 1022, 1023], np.int32)
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    Ys = [(torch.randn((T, E), generator=g, device="cuda") * (1 + 50 * (i == 1))).to(torch.bfloat16)
          for i in range(N)]
    w = dataclasses.replace(wl.TINY, N=N, T=T, E=E, k=idx.size, G=G)
    _codec_case(w, Ys, idx)


@pytest.mark.parametrize("name,cols", [
    ("one_odd_shift", [3]),                                   # every later chunk starts on an odd column
    ("run_in_the_middle", list(range(100, 121))),             # a chunk whose features lie 21 columns apart
    ("run_at_the_end", list(range(2048 - 12, 2048))),
    ("run_at_the_start", list(range(0, 12))),
    ("every_other", list(range(200, 264, 2))),                # four selected columns inside each chunk
    ("every_third", list(range(601, 700, 3))),
    ("across_pass_boundaries", list(range(505, 521)) + [1033, 1034, 1040, 1551]),
    ("last_column_only", [2047]),
    ("first_column_only", [0]),
    ("pairs", [c for b in range(64, 1900, 97) for c in (b, b + 1)]),
])
def test_outlier_patterns(name, cols):
    """Index sets that exercise every way a chunk can be cut (slots, second windows,
    features and selected columns out of a slot's reach)."""
    E, G, T, N = 2048, 128, 3, 2
    idx = np.array(sorted(set(cols)), np.int32)
    g = torch.Generator(device="cuda")
    g.manual_seed(len(cols) * 7 + cols[0])
    Ys = []
    for i in range(N):
        x = torch.randn((T, E), generator=g, device="cuda")
        x[:, torch.as_tensor(idx.astype(np.int64), device="cuda")] *= 60.0
        Ys.append(x.to(torch.bfloat16))
    w = dataclasses.replace(wl.TINY, N=N, T=T, E=E, k=idx.size, G=G)
    _codec_case(w, Ys, idx)


@pytest.mark.parametrize("E,G,cols", [
    (5120, 128, [5 + 31 * i for i in range(80)]),                      # every slot of the row in its first segment
    (8192, 64, [3 + 11 * i for i in range(341)]),                      # two dense segments, two without a slot
    (8192, 128, [3 + 11 * i for i in range(300)] + list(range(3300, 3341))),  # ... with a chunk cut by a long run
    (8192, 64, [4000 + 9 * i for i in range(341)]),                    # dense from the middle of the row on
], ids=["llama_width_first_segment", "large_width_two_segments", "large_width_with_run", "large_width_from_middle"])
def test_segments_denser_than_the_slot_area(E, G, cols):
    """Selected features crowded into part of the row: a segment then has more cut chunks than
    the encoder's LDS area holds slots for, and gathers the rest from memory."""
    T, N = 5, 2
    idx = np.array(sorted(set(cols)), np.int32)
    g = torch.Generator(device="cuda")
    g.manual_seed(E + len(cols))
    Ys = []
    for i in range(N):
        x = torch.randn((T, E), generator=g, device="cuda")
        x[:, torch.as_tensor(idx.astype(np.int64), device="cuda")] *= 40.0
        Ys.append(x.to(torch.bfloat16))
    w = dataclasses.replace(wl.TINY, N=N, T=T, E=E, k=idx.size, G=G)
    _codec_case(w, Ys, idx)


def test_denormal_and_huge_values():
    E, G, T = 512, 128, 4
    x = torch.zeros((T, E), device="cuda")
    x[0, :256] = 1e-39          # below the smallest normal: vanishing range
    x[0, 256:] = torch.linspace(-1e-38, 1e-38, 256, device="cuda")
    x[1] = torch.linspace(-3e37, 3e37, E, device="cuda")
    x[2] = torch.linspace(1e-20, 2e-20, E, device="cuda")
    x[3, ::2] = 65504.0
    Ys = [x.to(torch.bfloat16), (x * 0.5).to(torch.bfloat16)]
    idx = np.array([7, 300], np.int32)
    w = dataclasses.replace(wl.TINY, N=2, T=T, E=E, k=2, G=G)
    _codec_case(w, Ys, idx)


def test_plan_tables_and_bad_indices():
    E, k, G = 1024, 16, 128
    L = tpq.layout_init(E, k, G)
    rng = np.random.default_rng(0)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    plan = gpu_plan(L, idx)
    raw = plan.cpu().numpy()
    hdr = raw[:64].view(np.int32)
    assert hdr[2] == E and hdr[3] == k and hdr[4] == G and hdr[5] == E - k
    idx_off, src_off = hdr[8], hdr[9]
    assert np.array_equal(raw[idx_off: idx_off + 4 * k].view(np.int32), idx)
    src = raw[src_off: src_off + 2 * (E - k)].view(np.uint16)
    assert np.array_equal(src, compaction(idx, E).astype(np.uint16))
    # unsorted / duplicate / out-of-range index sets are refused and nothing is written
    y = [torch.randn((4, E), device="cuda").to(torch.bfloat16)]
    for bad in (idx[::-1].copy(), np.r_[idx[:-1], idx[-2]].astype(np.int32),
                np.r_[idx[:-1], E].astype(np.int32), np.r_[-1, idx[1:]].astype(np.int32)):
        bad_dev = torch.from_numpy(np.ascontiguousarray(bad)).cuda()
        p = tpq.plan_build(L, bad_dev)
        with pytest.raises(tpq.TpqError) as e:
            tpq.plan_check(L, p)
        assert e.value.code == tpq.ERR_INDEX
        msgs = gpu_encode(L, p, y)
        for t in (msgs[0].codes, msgs[0].scale, msgs[0].zero, msgs[0].outl):
            assert bool((t == CANARY).all().item())
        out = torch.full((4, E), 3.0, dtype=torch.bfloat16, device="cuda")
        tpq.decode_reduce(L, p, msgs, out)
        torch.cuda.synchronize()
        assert bool((out == 3.0).all().item())
    # a plan for another layout is refused as well
    L2 = tpq.layout_init(E, k, 64)
    with pytest.raises(tpq.TpqError):
        tpq.plan_check(L2, plan)


@pytest.mark.parametrize("E,cols", [
    (2048, [3, 100, 101, 102, 700, 705, 1029, 2047]),
    (1032, [0]),
    (520, list(range(1, 520, 9))),                 # every run is 8 features long
    (1024, list(range(4, 1024, 7))),               # every run is shorter than 8: narrow entries only
    (4096, []),
])
def test_plan_store_blocks(E, cols):
    """The decoder's store table against its definition: per pass of 512 compacted features,
    runs of consecutive columns; a run of 8 or more is covered by blocks of 8 (the last one
    aligned to the run's end), shorter runs feature by feature."""
    idx = np.array(cols, np.int32)
    k = idx.size
    L = tpq.layout_init(E, k, 128)
    raw = gpu_plan(L, idx).cpu().numpy()
    hdr = raw[:128].view(np.int32)
    spass_off, sblk_off, cap = hdr[23], hdr[24], hdr[25]
    src = compaction(idx, E)
    r = E - k
    passes = (r + 511) // 512
    spass = raw[spass_off: spass_off + 16 * passes].view(np.uint32).reshape(passes, 4)
    sblk = raw[sblk_off: sblk_off + 4 * cap].view(np.uint32)
    at = 0
    for p in range(passes):
        feats = src[512 * p: min(512 * (p + 1), r)]
        cuts = [0] + [i for i in range(1, feats.size) if feats[i] != feats[i - 1] + 1] + [feats.size]
        blocks, narrow = [], []
        for rs, re in zip(cuts[:-1], cuts[1:]):
            if re - rs >= 8:
                for a0 in range(rs, re, 8):
                    a = a0 if a0 + 8 <= re else re - 8
                    blocks.append(int(feats[a]) | (a << 16))
            else:
                narrow += [int(feats[a]) | (a << 16) for a in range(rs, re)]
        assert list(spass[p]) == [at, len(blocks), len(narrow), 0]
        assert list(sblk[at: at + len(blocks) + len(narrow)]) == blocks + narrow
        at += len(blocks) + len(narrow)
    assert at <= cap


def test_determinism():
    w = dataclasses.replace(wl.LLAMA_PREFILL, T=64)
    Ys = wl.partial_sums(w, device="cuda")
    idx = idx_for(w)
    L = tpq.layout_init(w.E, w.k, w.G)
    plan = gpu_plan(L, idx)
    first = None
    for _ in range(20):
        msgs = gpu_encode(L, plan, Ys)
        out, _ = gpu_decode(L, plan, msgs, w.T, tpq.ACC_FP32, False)
        blob = (out.tobytes(), *[m.codes.cpu().numpy().tobytes() for m in msgs])
        if first is None:
            first = blob
        assert blob == first


def test_hardware_behaviour_probe():
    """The instruction behaviour the kernels rely on for bit-exact results (rounding of the
    byte and bf16 conversions, the two division shortcuts checked against IEEE division --
    the reciprocal for every bf16 scale --, lane order of the DPP shift, byte order of the
    permute), checked by a stand-alone program that build() compiles."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "probes", "hw_probe")
    assert os.path.exists(exe), "tests/probes/hw_probe is not built: run __graft_entry__.build()"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0 and "HW PROBE OK" in r.stdout, r.stdout + r.stderr


def _sample_rows(T, n, seed):
    rng = np.random.default_rng(seed)
    rows = set(rng.choice(T, min(n, T), replace=False).tolist()) | {0, T - 1, T // 2}
    return np.array(sorted(rows), np.int64)


def test_llama_prefill_full_size():
    """The benchmark's configuration: every row of every rank checked against the oracle."""
    w = wl.LLAMA_PREFILL
    Ys = wl.partial_sums(w, device="cuda")
    _codec_case(w, Ys, idx_for(w), modes=((tpq.ACC_BF16, False), (tpq.ACC_FP32, False), (tpq.ACC_FAST, False)))


def test_gemma_decode_blocks():
    """Small-message regime: several blocks, each with its own outlier set."""
    w = wl.GEMMA_DECODE
    for block in (0, 1, 45, 91):
        Ys = wl.partial_sums(w, block=block, device="cuda")
        _codec_case(w, Ys, idx_for(w, block), modes=((tpq.ACC_BF16, False),))


@pytest.mark.parametrize("w", wl.large_variants(), ids=lambda w: w.name)
def test_large_prefill_variants(w):
    """N = 16, [16384 x 8192]: group 64 / 128, k for 4.2 / 4.5 bits, fp32 accumulate."""
    Ys = wl.partial_sums(w, device="cuda")
    _codec_case(w, Ys, idx_for(w), rows=_sample_rows(w.T, 1024, 2),
                modes=((tpq.ACC_FP32, True), (tpq.ACC_FP32, False)))
    del Ys
    torch.cuda.empty_cache()


# ---- calibration -------------------------------------------------------------------

def _calibrate_both(w, n_seq, S, block=0, N=None, gamma=0.01, ld_pad=0):
    N = w.N if N is None else N
    E = w.E
    m = torch.full((N, E), 9.0, device="cuda")
    M = torch.full((N, E), -9.0, device="cuda")
    ws = torch.zeros(tpq.calibrate_workspace_bytes(S, E), dtype=torch.uint8, device="cuda")
    m_ref = np.zeros((N, E), np.float32)
    M_ref = np.zeros((N, E), np.float32)
    for i in range(N):
        for s in range(n_seq):
            Y = wl.calibration_sequence(w, block, i, s, device="cuda", S=S)
            if ld_pad:
                buf = torch.full((S, E + ld_pad), 1e30, dtype=torch.bfloat16, device="cuda")
                buf[:, :E] = Y
                Yv = buf[:, :E]
            else:
                Yv = Y
            tpq.calibrate(Yv, i, N, s, gamma, m, M, ws)
            oracle.calibrate_update(wl.to_bits(Y), m_ref[i], M_ref[i], first=(s == 0), gamma=gamma)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy(), m_ref) and np.array_equal(M.cpu().numpy(), M_ref)
    return m, M, m_ref, M_ref


def _finalize_both(m, M, m_ref, M_ref, k):
    N, E = m_ref.shape
    R = torch.empty((N, E), device="cuda")
    Rbar = torch.empty(E, device="cuda")
    idx_s = torch.full((max(k, 1),), -7, dtype=torch.int32, device="cuda")
    idx_r = torch.full((max(k, 1),), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(tpq.calibrate_finalize_workspace_bytes(E), dtype=torch.uint8, device="cuda")
    tpq.calibrate_finalize(m, M, k, Rbar, idx_s, idx_r, ws, R=R)
    torch.cuda.synchronize()
    R_ref, Rbar_ref, s_ref, r_ref = oracle.calibrate_finalize(m_ref, M_ref, k)
    assert np.array_equal(R.cpu().numpy(), R_ref)
    assert np.array_equal(Rbar.cpu().numpy(), Rbar_ref)
    assert np.array_equal(idx_s.cpu().numpy()[:k], s_ref)
    assert np.array_equal(idx_r.cpu().numpy()[:k], r_ref)
    return idx_s[:k]


def test_calibrate_tiny_then_codec_end_to_end():
    """Calibrate -> select -> plan -> encode -> decode_reduce, all on the device."""
    w = wl.TINY
    m, M, m_ref, M_ref = _calibrate_both(w, wl.n_cal_sequences(w), w.cal_seq)
    idx_dev = _finalize_both(m, M, m_ref, M_ref, w.k)
    cols, _ = wl.outlier_columns(w)
    assert set(cols.tolist()) == set(idx_dev.cpu().tolist())
    Ys = wl.partial_sums(w, device="cuda")
    _codec_case(w, Ys, idx_dev.cpu().numpy().astype(np.int32))


@pytest.mark.parametrize("S,E,N,n_seq,ld_pad", [(1, 64, 2, 3, 0), (37, 520, 3, 4, 8),
                                                (256, 5120, 2, 3, 0), (1000, 4608, 2, 2, 24)])
def test_calibrate_shapes(S, E, N, n_seq, ld_pad):
    w = dataclasses.replace(wl.CALIBRATION, E=E, N=N)
    m, M, m_ref, M_ref = _calibrate_both(w, n_seq, S, ld_pad=ld_pad)
    for k in (0, 1, E // 64, E):
        _finalize_both(m, M, m_ref, M_ref, k)


def test_calibrate_ties_and_gamma():
    E, N = 512, 2
    m = -torch.ones((N, E), device="cuda")
    M = torch.ones((N, E), device="cuda")
    M[:, 100] = 4.0
    _finalize_both(m, M, m.cpu().numpy(), M.cpu().numpy(), 8)
    w = dataclasses.replace(wl.CALIBRATION, E=E, N=N)
    _calibrate_both(w, 3, 50, gamma=1.0)
    _calibrate_both(w, 3, 50, gamma=0.25)


def test_calibration_config_reduced_stream_and_resume():
    """Gemma-shaped calibration: 16384-token chunks; a reduced stream per block, and
    stop / copy state / resume gives the same bits as running straight through."""
    w = wl.CALIBRATION
    for block in (0, 91):
        m, M, m_ref, M_ref = _calibrate_both(w, 3, w.cal_seq, block=block, N=2)
        idx = _finalize_both(m, M, m_ref, M_ref, w.k)
        cols, _ = wl.outlier_columns(w, block)
        assert set(cols.tolist()) <= set(idx.cpu().tolist())
    # resume
    S, N, E = 4096, 1, w.E
    ws = torch.zeros(tpq.calibrate_workspace_bytes(S, E), dtype=torch.uint8, device="cuda")
    seqs = [wl.calibration_sequence(w, 3, 0, s, device="cuda", S=S) for s in range(6)]
    mA, MA = torch.zeros((N, E), device="cuda"), torch.zeros((N, E), device="cuda")
    for s, Y in enumerate(seqs):
        tpq.calibrate(Y, 0, N, s, 0.01, mA, MA, ws)
    mB, MB = torch.zeros((N, E), device="cuda"), torch.zeros((N, E), device="cuda")
    for s, Y in enumerate(seqs[:3]):
        tpq.calibrate(Y, 0, N, s, 0.01, mB, MB, ws)
    mC, MC = mB.cpu().cuda(), MB.cpu().cuda()      # checkpoint = the two arrays
    for s, Y in enumerate(seqs[3:], start=3):
        tpq.calibrate(Y, 0, N, s, 0.01, mC, MC, ws)
    torch.cuda.synchronize()
    assert torch.equal(mA, mC) and torch.equal(MA, MC)


def test_calibration_config_full_stream_one_block():
    """All 64 chunks of 16384 tokens of one (block, rank) of the calibration configuration:
    the moving averages after every chunk equal the oracle's, bit for bit."""
    w = wl.CALIBRATION
    E, S = w.E, w.cal_seq
    n_chunks = 64
    m = torch.zeros((1, E), device="cuda")
    M = torch.zeros((1, E), device="cuda")
    ws = tpq.calibrate_workspace(S, E, "cuda")
    m_ref = np.zeros((1, E), np.float32)
    M_ref = np.zeros((1, E), np.float32)
    for s in range(n_chunks):
        Y = wl.calibration_sequence(w, 7, 3, s, device="cuda")
        tpq.calibrate(Y, 0, 1, s, 0.01, m, M, ws)
        oracle.calibrate_update(wl.to_bits(Y), m_ref[0], M_ref[0], first=(s == 0), gamma=0.01)
        if s in (0, 1, 15, 63):
            assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref.view(np.uint32)), s
            assert np.array_equal(M.cpu().numpy().view(np.uint32), M_ref.view(np.uint32)), s


def test_finalize_sweep_over_blocks():
    """Range aggregation and top-k of many blocks from oracle-made states (no 16384-row data
    needed): Rbar, both index lists and the planted columns, bit for bit."""
    w = wl.CALIBRATION
    rng = np.random.default_rng(11)
    for block in range(0, w.blocks, 7):
        cols, _ = wl.outlier_columns(w, block)
        m_ref = -np.abs(rng.standard_normal((w.N, w.E))).astype(np.float32) * 4
        M_ref = np.abs(rng.standard_normal((w.N, w.E))).astype(np.float32) * 4
        M_ref[:, cols.numpy()] *= 40.0
        ties = np.setdiff1d(np.arange(0, w.E, 501), cols.numpy())
        m_ref[:, ties] = 0.0                               # ties at zero range
        M_ref[:, ties] = 0.0
        m = torch.from_numpy(m_ref).cuda()
        M = torch.from_numpy(M_ref).cuda()
        idx = _finalize_both(m, M, m_ref, M_ref, w.k)
        assert set(cols.tolist()) <= set(idx.cpu().tolist())


def test_hip_graph_replays_match_eager():
    """encode + decode_reduce of several blocks captured in one HIP graph: every replay, with
    eager work and synchronisation in between, gives the eager result."""
    w = wl.TINY
    L = tpq.layout_init(w.E, w.k, w.G)
    plan = gpu_plan(L, idx_for(w))
    blocks = []
    for b in range(3):
        Ys = wl.partial_sums(w, block=b, device="cuda")
        msgs = [tpq.Message(L, w.T, "cuda") for _ in range(w.N)]
        out = torch.empty((w.T, w.E), dtype=torch.bfloat16, device="cuda")
        bias = torch.linspace(-1, 1, w.E, device="cuda").to(torch.bfloat16)
        blocks.append(dict(enc=tpq.encode_call(L, plan, Ys, msgs),
                           dec=tpq.decode_reduce_fused_call(L, plan, msgs, out, None, bias, tpq.ACC_BF16),
                           out=out, msgs=msgs, keep=(Ys, bias)))
    calls = [c for blk in blocks for c in (blk["enc"], blk["dec"])]
    for c in calls:
        c()
    torch.cuda.synchronize()
    eager = [blk["out"].clone() for blk in blocks]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for c in calls:
            c()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for c in calls:
            c()
    for rep in range(4):
        for blk in blocks:                      # eager work between the replays
            blk["out"].fill_(3.0)
            for m in blk["msgs"]:
                m.codes.fill_(0x5A)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for blk, e in zip(blocks, eager):
            assert torch.equal(blk["out"], e), "replay %d differs from the eager result" % rep


def test_timing_events_on_a_launch():
    """tpq_bench_time_next_launch: the events bracket the next kernel only; results are unchanged."""
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    idx = idx_for(w)
    L = tpq.layout_init(w.E, w.k, w.G)
    plan = gpu_plan(L, idx)
    plain = gpu_encode(L, plan, Ys)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    timed = [tpq.Message(L, w.T, "cuda", fill=CANARY) for _ in Ys]
    out = torch.empty((w.T, w.E), dtype=torch.bfloat16, device="cuda")
    tpq.bench_time_next_launch(ev[0], ev[1])
    tpq.encode(L, plan, Ys, timed)
    tpq.bench_time_next_launch(ev[2], ev[3])
    tpq.decode_reduce(L, plan, timed, out, tpq.ACC_BF16)
    tpq.decode_reduce(L, plan, timed, out, tpq.ACC_BF16)   # no request pending: a plain launch
    torch.cuda.synchronize()
    for a, b in zip(plain, timed):
        for name in ("codes", "scale", "zero", "outl"):
            assert torch.equal(getattr(a, name), getattr(b, name))
    assert 0.0 < ev[0].elapsed_time(ev[1]) < 50.0
    assert 0.0 < ev[2].elapsed_time(ev[3]) < 50.0
    tpq.bench_time_next_launch(ev[0], ev[1])
    tpq.bench_time_next_launch(None, None)                       # cancelled
    lib = tpq._load()
    assert lib.tpq_bench_time_next_launch(ev[0].cuda_event, None) == tpq.ERR_NULL
