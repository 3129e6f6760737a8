"""Oracle of the stochastic similarity filter (Sec. 3.4, Eq. 8 and Eq. 9).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings where the paper is silent:
  * the image vector is all H*W*3 raw u8 values, no mean shift;
  * dot product and squared norms are exact integers; S_C = dot / sqrt(|I_t|^2 * |I_ref|^2) in float64, capped at 1;
  * eta >= 1 or a zero-norm frame gives P = 0; the first frame is never skipped and becomes the reference;
  * the uniform draw of frame k is u_k = (mix(seed + (k+1) * 0x9E3779B97F4A7C15) >> 11) * 2^-53 with mix the
    SplitMix64 output function (Steele, Lea & Flood 2014); one draw per frame index; skip iff u_k < P;
  * the reference is replaced only by frames that were not skipped;
  * the hard-threshold filter the paper compares against (note at the end of Sec. 3.4; user study, Table 3) skips
    exactly when S_C > eta, i.e. when Eq. 9 gives a positive probability, and draws nothing;
  * run statistics: duty cycle = processed frames / frames (the share of steps the GPU actually runs, the
    quantity behind the power measurement), longest run of consecutive skips (how long the output can stay stuck).
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
    def __init__(self, eta: float, seed: int, hard: bool = False):
        self.eta, self.seed, self.hard = float(eta), int(seed), bool(hard)
        self.ref: Optional[np.ndarray] = None

    def __call__(self, frame: np.ndarray, k: int) -> Tuple[bool, float]:
        """Returns (skip, P) for frame index k and updates the reference when the frame is let through.
        With hard=True the second value is the similarity S_C (0 while there is no reference)."""
        if self.ref is None:
            s_c, has_ref = 0.0, False
        else:
            d, nt, nr = sums(frame, self.ref)
            has_ref = not (nt == 0 or nr == 0)
            s_c = cosine(d, nt, nr)
        if self.hard:
            skip, val = has_ref and s_c > self.eta, s_c
        else:
            p = skip_probability(s_c, self.eta) if has_ref else 0.0
            skip, val = uniform(self.seed, k) < p, p
        if not skip:
            self.ref = frame.copy()
        return skip, val


def run_statistics(skips) -> dict:
    """skips: one bool per frame in order."""
    skips = [bool(v) for v in skips]
    longest = cur = 0
    for v in skips:
        cur = cur + 1 if v else 0
        longest = max(longest, cur)
    n = len(skips)
    return {"frames": n, "processed": n - sum(skips), "duty_cycle": (n - sum(skips)) / n if n else 0.0,
            "longest_skip_run": longest}
