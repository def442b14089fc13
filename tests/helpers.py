"""Test-side helpers: fixture parsing and slow reference computations written in plain
Python/NumPy.  Independent of both the oracle and the HIP library."""
import os
import struct
from fractions import Fraction

import numpy as np


def load_golden(path):
    """`name: v0 v1 ...` lines -> dict of float64 arrays (scalars as Python numbers)."""
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            name, vals = line.split(":", 1)
            nums = [float(v) for v in vals.split()]
            out[name.strip()] = nums[0] if name.strip() in ("n", "numel", "k", "step", "lr", "beta", "chunk") else np.array(nums)
    for key in ("n", "numel", "k", "step", "chunk"):
        if key in out:
            out[key] = int(out[key])
    return out


def mag_key(x) -> int:
    """Magnitude of a binary32 value as an integer: its bit pattern without the sign."""
    return struct.unpack("<I", struct.pack("<f", float(x)))[0] & 0x7FFFFFFF


def brute_topk(x, k):
    """Eq. 2 with ties resolved by position: sort every position by (magnitude descending,
    position ascending) in pure Python and keep the first k."""
    order = sorted(range(len(x)), key=lambda j: (-mag_key(x[j]), j))
    return np.array(sorted(order[:k]), dtype=np.int32)


def round_fraction_to_f32(fr: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 value of an exact rational."""
    if fr == 0:
        return np.float32(0.0)
    guess = np.float32(float(fr))
    cands = {guess, np.nextafter(guess, np.float32(np.inf)), np.nextafter(guess, np.float32(-np.inf))}
    best = None
    for c in cands:
        if not np.isfinite(c):
            continue
        d = abs(Fraction(float(c)) - fr)
        even = (struct.unpack("<I", struct.pack("<f", float(c)))[0] & 1) == 0
        keyc = (d, 0 if even else 1)
        if best is None or keyc < best[0]:
            best = (keyc, c)
    return best[1]


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even truncation of float32 to bfloat16 patterns (uint16), finite inputs."""
    b = a.astype(np.float32).view(np.uint32).astype(np.uint64)
    rounded = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32)
