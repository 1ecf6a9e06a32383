"""Synthetic static-camera video.

A frame is  background  (+ textured rectangles pasted at their current position)
(+ fresh Gaussian noise), planar [C][H][W] float32, values around [0, 1], never clipped.
It stands in for the surveillance sequences of the paper's evaluation (Section 4.1),
where moving objects cover a small part of an otherwise static scene (Fig. 3).

Every frame is a pure function of (seeds, t): frames can be produced in any order and
regenerated on another machine bit-for-bit (numpy PCG64 streams only).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([int(k) & 0xFFFFFFFF for k in key]))


def _reflect(p0: int, v: int, t: int, span: int) -> int:
    """Position at time t of a point starting at p0 with velocity v bouncing in [0, span]."""
    if span <= 0:
        return 0
    period = 2 * span
    u = (p0 + v * t) % period
    return u if u <= span else period - u


@dataclass
class MovingObject:
    y0: int
    x0: int
    h: int
    w: int
    vy: int
    vx: int
    texture: np.ndarray  # [C][h][w] float32, moves with the object

    def position(self, t: int, H: int, W: int) -> Tuple[int, int]:
        return (_reflect(self.y0, self.vy, t, H - self.h),
                _reflect(self.x0, self.vx, t, W - self.w))


class SyntheticVideo:
    """Static background + moving rectangles + per-frame noise.

    seeds: (background, objects, noise) integer seeds.
    objects: explicit list, or None to draw `n_objects` rectangles with side lengths
        uniform in size_range (inclusive) and per-axis speeds uniform in speed_range
        (inclusive) with a random sign.
    flicker: if True the background itself is redrawn for every frame (every pixel
        changes every frame: the worst case of Section 3.1, matrix multiplication paragraph).
    """

    def __init__(self, height: int, width: int, channels: int = 3, *,
                 seeds: Sequence[int], sigma: float = 0.0, n_objects: int = 0,
                 size_range: Tuple[int, int] = (10, 40), speed_range: Tuple[int, int] = (1, 4),
                 objects: Optional[List[MovingObject]] = None, flicker: bool = False):
        self.H, self.W, self.C = int(height), int(width), int(channels)
        self.sigma = float(sigma)
        self.flicker = bool(flicker)
        self.seed_bg, self.seed_obj, self.seed_noise = (int(s) for s in seeds)
        self.background = _rng(self.seed_bg).random((self.C, self.H, self.W), dtype=np.float32)
        if objects is not None:
            self.objects = list(objects)
        else:
            r = _rng(self.seed_obj)
            self.objects = []
            for _ in range(int(n_objects)):
                h = int(r.integers(size_range[0], size_range[1] + 1))
                w = int(r.integers(size_range[0], size_range[1] + 1))
                h, w = min(h, self.H), min(w, self.W)
                y0 = int(r.integers(0, self.H - h + 1))
                x0 = int(r.integers(0, self.W - w + 1))
                vy = int(r.integers(speed_range[0], speed_range[1] + 1)) * (1 if r.random() < 0.5 else -1)
                vx = int(r.integers(speed_range[0], speed_range[1] + 1)) * (1 if r.random() < 0.5 else -1)
                tex = r.random((self.C, h, w), dtype=np.float32)
                self.objects.append(MovingObject(y0, x0, h, w, vy, vx, tex))

    def clean_frame(self, t: int) -> np.ndarray:
        """Frame t without sensor noise."""
        if self.flicker:
            f = _rng(self.seed_bg, 7, t).random((self.C, self.H, self.W), dtype=np.float32)
        else:
            f = self.background.copy()
        for ob in self.objects:
            y, x = ob.position(t, self.H, self.W)
            f[:, y:y + ob.h, x:x + ob.w] = ob.texture
        return f

    def frame(self, t: int) -> np.ndarray:
        f = self.clean_frame(t)
        if self.sigma > 0.0:
            n = _rng(self.seed_noise, t).standard_normal((self.C, self.H, self.W), dtype=np.float32)
            f = f + np.float32(self.sigma) * n
        return np.ascontiguousarray(f, dtype=np.float32)

    def frames(self, n: int, start: int = 0) -> np.ndarray:
        return np.stack([self.frame(t) for t in range(start, start + n)])

    def moved_fraction(self, t: int) -> float:
        """Share of pixels whose noise-free value differs between frames t-1 and t
        (a property of the generated data; used only to describe a workload)."""
        a, b = self.clean_frame(t - 1), self.clean_frame(t)
        return float(np.any(a != b, axis=0).mean())
