"""Seeded synthetic inputs for the codec: partial sums and calibration streams.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds none of the method's arithmetic: it only draws random
activations of the shapes, value distributions and outlier structure of the
workloads (a few feature columns with an enormous range, as in the paper's
Fig. 1, the rest near unit scale) and converts between torch bf16 tensors and
raw uint16 bit patterns.  Real model activations (the paper calibrates on
WikiText sequences and evaluates Llama 2 13B / Gemma 2 27B / Mistral NeMo 12B
with tensor parallelism over 8 devices, Sec. 3-4) are not available; these
tensors stand in for them.

Everything is generated with a seeded ``torch.Generator`` on the requested
device.  The same tensor is handed to both sides of a parity test, so results do
not depend on the generator being portable between CPU and GPU.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np
import torch


# --------------------------------------------------------------------------
# bf16 <-> raw bits (format conversion only)
# --------------------------------------------------------------------------

def to_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor (any device) -> numpy uint16 array of its bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def from_bits(a: np.ndarray, device="cpu") -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 tensor."""
    assert a.dtype == np.uint16
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


def bits_to_f32(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 values (exact)."""
    return (a.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the list of benchmark configurations
    N: int                # simulated tensor-parallel devices
    T: int                # tokens (rows) per block
    E: int                # features (columns)
    k: int                # features kept in bf16
    G: int                # quantisation group size along compacted features
    base: str             # "normal" or "t3": distribution of ordinary columns
    outlier_frac: float   # fraction of columns planted as outliers
    outlier_std: tuple    # (lo, hi) of the per-column scale
    outlier_std_law: str  # "uniform" or "loguniform"
    outlier_noise: str    # "normal" or "t3": distribution of outlier-column entries
    rank_jitter: tuple = (1.0, 1.0)   # per-device multiplier range of an outlier column's scale
    sign_flip: bool = False           # random sign per (token, outlier column)
    fixed_scale: Optional[float] = None  # if set, outlier columns are base * this value
    accum: str = "bf16"   # accumulate mode the workload is quoted with
    out_dtype: str = "bf16"
    blocks: int = 1       # attention / feed-forward blocks with their own outlier sets
    cal_tokens: int = 0   # calibration tokens per device
    cal_seq: int = 0      # tokens per calibration sequence (one EMA update each)
    seed: Optional[int] = None

    @property
    def r(self) -> int:
        return self.E - self.k

    @property
    def n_outlier_cols(self) -> int:
        return max(1, int(round(self.outlier_frac * self.E))) if self.outlier_frac > 0 else 0


TINY = Workload("tiny", 0, N=4, T=16, E=512, k=8, G=128, base="normal",
                outlier_frac=8 / 512, outlier_std=(50.0, 50.0), outlier_std_law="uniform",
                outlier_noise="normal", fixed_scale=50.0, accum="bf16",
                cal_tokens=256, cal_seq=64, seed=0)

LLAMA_PREFILL = Workload("llama2_13b_prefill", 1, N=8, T=2048, E=5120, k=80, G=128, base="normal",
                         outlier_frac=0.005, outlier_std=(30.0, 100.0), outlier_std_law="uniform",
                         outlier_noise="t3", rank_jitter=(0.5, 1.5), accum="bf16",
                         cal_tokens=4096, cal_seq=256)

GEMMA_DECODE = Workload("gemma2_27b_decode", 2, N=8, T=64, E=4608, k=72, G=128, base="normal",
                        outlier_frac=0.01, outlier_std=(20.0, 200.0), outlier_std_law="loguniform",
                        outlier_noise="normal", accum="bf16", blocks=92)

CALIBRATION = Workload("gemma2_27b_calibration", 3, N=8, T=16384, E=4608, k=72, G=128, base="normal",
                       outlier_frac=0.01, outlier_std=(10.0, 300.0), outlier_std_law="loguniform",
                       outlier_noise="normal", blocks=92, cal_tokens=1048576, cal_seq=16384)

LARGE_PREFILL = Workload("large_prefill", 4, N=16, T=16384, E=8192, k=128, G=128, base="t3",
                         outlier_frac=0.0025, outlier_std=(50.0, 500.0), outlier_std_law="loguniform",
                         outlier_noise="t3", sign_flip=True, accum="fp32", out_dtype="fp32")


def large_variants() -> List[Workload]:
    """The four (group size) x (bits) variants of the large prefill stress case."""
    out = []
    for k, tag in ((128, "4p2"), (341, "4p5")):
        for G in (128, 64):
            out.append(replace(LARGE_PREFILL, name=f"large_prefill_{tag}_g{G}", k=k, G=G))
    return out


ALL = [TINY, LLAMA_PREFILL, GEMMA_DECODE, CALIBRATION, LARGE_PREFILL]


def seed_for(w: Workload, block: int, rank: int, stream: int = 0) -> int:
    """Seed = 1000*config + 10*block + rank (+ a stream offset), or the fixed one."""
    base = w.seed if w.seed is not None else 1000 * w.index
    return base * 1_000_003 + 10 * block + rank + 7919 * stream


# --------------------------------------------------------------------------
# random draws
# --------------------------------------------------------------------------

def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _student_t3(shape, g: torch.Generator, device) -> torch.Tensor:
    z = torch.randn(shape, generator=g, device=device)
    v = torch.zeros(shape, device=device)
    for _ in range(3):
        v += torch.randn(shape, generator=g, device=device) ** 2
    return z / torch.sqrt(v / 3.0)


def _draw(kind: str, shape, g, device) -> torch.Tensor:
    if kind == "normal":
        return torch.randn(shape, generator=g, device=device)
    if kind == "t3":
        return _student_t3(shape, g, device)
    raise ValueError(kind)


def outlier_columns(w: Workload, block: int = 0):
    """The planted outlier columns of a block and their scales (shared by all devices)."""
    g = _gen("cpu", seed_for(w, block, 0, stream=1))
    n = w.n_outlier_cols
    cols = torch.randperm(w.E, generator=g)[:n].sort().values
    lo, hi = w.outlier_std
    u = torch.rand(n, generator=g)
    if w.outlier_std_law == "loguniform":
        std = torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
    else:
        std = lo + u * (hi - lo)
    return cols, std


def _rows(w: Workload, T: int, block: int, rank: int, stream: int, device) -> torch.Tensor:
    g = _gen(device, seed_for(w, block, rank, stream=stream))
    x = _draw(w.base, (T, w.E), g, device)
    cols, std = outlier_columns(w, block)
    n = cols.numel()
    if n:
        gc = _gen("cpu", seed_for(w, block, rank, stream=2))
        jl, jh = w.rank_jitter
        jitter = jl + (jh - jl) * torch.rand(n, generator=gc)
        if w.fixed_scale is not None:
            x[:, cols.to(device)] *= w.fixed_scale
        else:
            o = _draw(w.outlier_noise, (T, n), g, device) * (std * jitter).to(device)
            if w.sign_flip:
                sign = torch.randint(0, 2, (T, n), generator=g, device=device) * 2 - 1
                o = o * sign
            x[:, cols.to(device)] = o
    return x.to(torch.bfloat16)


def partial_sums(w: Workload, block: int = 0, device="cpu", T: Optional[int] = None,
                 ranks: Optional[range] = None) -> List[torch.Tensor]:
    """The N devices' row-parallel partial sums of one block: N bf16 tensors [T,E]."""
    T = w.T if T is None else T
    ranks = range(w.N) if ranks is None else ranks
    return [_rows(w, T, block, i, 0, device) for i in ranks]


def calibration_sequence(w: Workload, block: int, rank: int, seq: int, device="cpu",
                         S: Optional[int] = None) -> torch.Tensor:
    """One calibration sequence (S tokens) of one device: bf16 [S,E]."""
    S = (w.cal_seq or w.T) if S is None else S
    return _rows(w, S, block, rank, 100 + seq, device)


def n_cal_sequences(w: Workload) -> int:
    return w.cal_tokens // w.cal_seq if w.cal_seq else 0


def linear_inputs(T: int, K: int, E: int, outlier_rows, seed: int, device="cpu", integer: bool = False):
    """Inputs of one device's row-parallel linear layer (Sec. 2): activations X bf16 [T,K] and
    the weight slice Wt bf16 [E,K], one row per output feature.  The rows in `outlier_rows` are
    scaled up so that those output features get the enormous range of the paper's Fig. 1.
    integer: small integers instead (every product and every partial sum is then exact in
    fp32, whatever the order of the additions)."""
    g = _gen(device, 7_000_003 * int(seed) + 13 * T + 17 * K + 19 * E)
    if integer:
        X = torch.randint(-3, 4, (T, K), generator=g, device=device).to(torch.float32)
        Wt = torch.randint(-3, 4, (E, K), generator=g, device=device).to(torch.float32)
    else:
        X = torch.randn((T, K), generator=g, device=device)
        Wt = torch.randn((E, K), generator=g, device=device) / math.sqrt(K)
        rows = torch.as_tensor(np.asarray(outlier_rows, np.int64), device=device)
        if rows.numel():
            Wt[rows] *= 30.0
    return X.to(torch.bfloat16), Wt.to(torch.bfloat16)
