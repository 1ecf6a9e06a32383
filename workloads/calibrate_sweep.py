"""Find the object counts of the change-rate sweeps (SWEEP_OBJECTS and SWEEP320_OBJECTS in configs.py).

For each nominal rate, bisect on the number of rectangles until the mean share of pixels
whose noise-free value moves between consecutive frames (frames 1..8) reaches the rate.
Run:  python -m workloads.calibrate_sweep
"""
from __future__ import annotations

import numpy as np

from .configs import SEED_BASE
from .video import SyntheticVideo


def mean_moved(n_objects: int, height: int = 720, width: int = 1280, config: int = 3, frames=range(1, 9)) -> float:
    base = SEED_BASE + 1000 * config
    v = SyntheticVideo(height, width, 3, seeds=(base + 1, base + 2, base + 3), sigma=0.0, n_objects=n_objects)
    return float(np.mean([v.moved_fraction(t) for t in frames]))


def calibrate(rate: float, nearest: bool = False, **kw) -> int:
    """Smallest object count whose moved share reaches the rate; nearest=True: of that count and the
    one below it, the one whose share is closer to the rate in ratio (small frames, where one object
    more is a large step)."""
    lo, hi = 0, 1
    while mean_moved(hi, **kw) < rate:
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if mean_moved(mid, **kw) < rate:
            lo = mid
        else:
            hi = mid
    if nearest and lo > 0 and rate / mean_moved(lo, **kw) < mean_moved(hi, **kw) / rate:
        return lo
    return hi


if __name__ == "__main__":
    for rate in (0.005, 0.02, 0.10, 0.30):
        n = calibrate(rate)
        print("1280x720 rate %.3f -> %d objects (measured %.4f)" % (rate, n, mean_moved(n)))
    for rate in (0.01, 0.05, 0.20):
        kw = dict(height=240, width=320, config=2)
        n = calibrate(rate, nearest=True, **kw)
        print("320x240 rate %.3f -> %d objects (measured %.4f)" % (rate, n, mean_moved(n, **kw)))
