"""Oracle of the stochastic similarity filter (Sec. 3.4, Eq. 8 and Eq. 9).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings where the paper is silent:
  * the image vector is all H*W*3 raw u8 values, no mean shift;
  * dot product and squared norms are exact integers; S_C = dot / sqrt(|I_t|^2 * |I_ref|^2) in float64, capped at 1;
  * eta >= 1 or a zero-norm frame gives P = 0; the first frame is never skipped and becomes the reference;
  * the uniform draw of frame k is u_k = (mix(seed + (k+1) * 0x9E3779B97F4A7C15) >> 11) * 2^-53 with mix the
    SplitMix64 output function (Steele, Lea & Flood 2014); one draw per frame index; skip iff u_k < P;
  * the reference is replaced only by frames that were not skipped.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

M64 = (1 << 64) - 1


def splitmix64_mix(z: int) -> int:
    z &= M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def uniform(seed: int, k: int) -> float:
    z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & M64
    return (splitmix64_mix(z) >> 11) * (2.0 ** -53)


def sums(frame: np.ndarray, ref: np.ndarray) -> Tuple[int, int, int]:
    f = frame.reshape(-1).astype(np.int64)
    r = ref.reshape(-1).astype(np.int64)
    return int((f * r).sum()), int((f * f).sum()), int((r * r).sum())


def cosine(dot: int, n_t: int, n_ref: int) -> float:
    """Eq. 8."""
    if n_t == 0 or n_ref == 0:
        return 0.0
    return min(float(dot) / math.sqrt(float(n_t) * float(n_ref)), 1.0)


def skip_probability(s_c: float, eta: float) -> float:
    """Eq. 9."""
    if eta >= 1.0:
        return 0.0
    return max(0.0, (s_c - eta) / (1.0 - eta))


class Filter:
    def __init__(self, eta: float, seed: int):
        self.eta, self.seed = float(eta), int(seed)
        self.ref: Optional[np.ndarray] = None

    def __call__(self, frame: np.ndarray, k: int) -> Tuple[bool, float]:
        """Returns (skip, P) for frame index k and updates the reference when the frame is let through."""
        u = uniform(self.seed, k)
        if self.ref is None:
            p = 0.0
        else:
            d, nt, nr = sums(frame, self.ref)
            p = 0.0 if (nt == 0 or nr == 0) else skip_probability(cosine(d, nt, nr), self.eta)
        skip = u < p
        if not skip:
            self.ref = frame.copy()
        return skip, p
