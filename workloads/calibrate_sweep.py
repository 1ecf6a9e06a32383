"""Find the object counts of the 1280x720 change-rate sweep (SWEEP_OBJECTS in configs.py).

For each nominal rate, bisect on the number of rectangles until the mean share of pixels
whose noise-free value moves between consecutive frames (frames 1..8) reaches the rate.
Run:  python -m workloads.calibrate_sweep
"""
from __future__ import annotations

import numpy as np

from .configs import SEED_BASE
from .video import SyntheticVideo


def mean_moved(n_objects: int, frames=range(1, 9)) -> float:
    v = SyntheticVideo(720, 1280, 3, seeds=(SEED_BASE + 3001, SEED_BASE + 3002, SEED_BASE + 3003),
                       sigma=0.0, n_objects=n_objects)
    return float(np.mean([v.moved_fraction(t) for t in frames]))


def calibrate(rate: float) -> int:
    lo, hi = 0, 1
    while mean_moved(hi) < rate:
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if mean_moved(mid) < rate:
            lo = mid
        else:
            hi = mid
    return hi


if __name__ == "__main__":
    for rate in (0.005, 0.02, 0.10, 0.30):
        n = calibrate(rate)
        print("rate %.3f -> %d objects (measured %.4f)" % (rate, n, mean_moved(n)))
