"""Independent numpy helpers for pinning the oracle.

Nothing here calls the oracle or the GPU library.  These are the plain
definitions (float64 brute force, closed forms, library conversions) that the
oracle's outputs are checked against.
"""
import numpy as np
import torch


def bits_to_f32(a):
    return (np.asarray(a, np.uint16).astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits_lib(x):
    """float32 -> bf16 bits through torch's own conversion (round-nearest-even)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def f32_vals_to_bits(x):
    """bf16-representable float values -> bit patterns (asserts exactness)."""
    x = np.asarray(x, np.float32)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not representable in bf16"
    return (u >> 16).astype(np.uint16)


def compaction(idx, E):
    """Feature index of each non-selected feature, ascending."""
    mask = np.ones(E, bool)
    mask[np.asarray(idx, np.int64)] = False
    return np.nonzero(mask)[0]


def unpack_codes(codes, r):
    """[T,cb] bytes -> [T,r] codes; byte b holds code 2b (low nibble), 2b+1 (high)."""
    codes = np.asarray(codes, np.uint8)
    lo = codes & 0x0F
    hi = codes >> 4
    both = np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)
    return both[:, :r], both[:, r:]


def group_expand(a, G, r):
    """[T,ng] per-group values -> [T,r] per-element."""
    return np.repeat(a, G, axis=1)[:, :r]


def payload_bits(E, k):
    return (16 * k + 4 * (E - k)) / E


def wire_bytes_per_row(E, k, G):
    r = E - k
    return 2 * k + (r + 1) // 2 + 4 * ((r + G - 1) // G)
