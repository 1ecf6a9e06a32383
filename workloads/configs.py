"""The five benchmark workloads, as seeded recipes.

seed = SEED_BASE + 1000*config + k  with k = 0 weights, 1 background, 2 objects, 3 noise;
multi-stream workloads add 10*stream to k = 1..3.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from .networks import (LayerSpec, make_weights, scene_labeling_net, single_layer_net, strided_net, vgg10_net)
from .video import MovingObject, SyntheticVideo, _rng

SEED_BASE = 170404313

# Object counts for the 1280x720 change-rate sweep.  Written by calibrate_sweep.py
# (beside this file): the smallest count whose mean share of moved pixels
# (SyntheticVideo.moved_fraction, noise-free) over frames 1..8 reaches the nominal rate.
SWEEP_OBJECTS: Dict[float, int] = {0.005: 6, 0.02: 23, 0.10: 126, 0.30: 445}
# The same for the 320x240 frames of the benchmark network, where one rectangle more is a large
# step: the count whose moved share is nearest to the nominal rate (measured 0.61 / 5.04 / 19.8 %).
SWEEP320_OBJECTS: Dict[float, int] = {0.01: 1, 0.05: 5, 0.20: 25}


@dataclass
class Config:
    name: str
    index: int
    layers: List[LayerSpec]
    height: int
    width: int
    channels: int
    n_frames: int
    tau: float
    sigma: float
    n_streams: int = 1
    dtype: str = "f32"
    video_kwargs: dict = field(default_factory=dict)

    def seed(self, k: int, stream: int = 0) -> int:
        return SEED_BASE + 1000 * self.index + k + (10 * stream if k else 0)

    def weights(self):
        return make_weights(self.layers, self.seed(0))

    def video(self, stream: int = 0) -> SyntheticVideo:
        kw = dict(self.video_kwargs)
        if "objects_fn" in kw:
            kw["objects"] = kw.pop("objects_fn")(self, stream)
        if "n_objects_fn" in kw:
            kw["n_objects"] = kw.pop("n_objects_fn")(self, stream)
        return SyntheticVideo(self.height, self.width, self.channels,
                              seeds=(self.seed(1, stream), self.seed(2, stream), self.seed(3, stream)),
                              sigma=self.sigma, **kw)


def _cfg1_objects(cfg: Config, stream: int):
    tex = _rng(cfg.seed(2, stream)).random((cfg.channels, 8, 8), dtype=np.float32)
    return [MovingObject(y0=28, x0=10, h=8, w=8, vy=0, vx=2, texture=tex)]


def _cfg5_count(cfg: Config, stream: int) -> int:
    return 1 + int(_rng(cfg.seed(2, stream), 99).integers(0, 4))


def get_config(index: int, *, height: Optional[int] = None, width: Optional[int] = None,
               n_frames: Optional[int] = None, sigma: Optional[float] = None,
               change_rate: Optional[float] = None, n_streams: Optional[int] = None) -> Config:
    """index 1..5 = the five workloads, 6 = a strided / mixed-filter-size network; the keyword arguments make reduced-size or
    swept replicas of the same recipe (same seeds)."""
    if index == 1:
        c = Config("cfg1-single-7x7", 1, single_layer_net(), 64, 64, 3, 8, 0.02, 0.005,
                   video_kwargs={"objects_fn": _cfg1_objects})
    elif index == 2 and change_rate is not None:
        # the benchmark network and frame size, noise-free, motion chosen per nominal change rate
        rate = float(change_rate)
        c = Config("cfg2-sweep-320x240-rate%g" % rate, 2, scene_labeling_net(), 240, 320, 3, 100, 0.02, 0.0,
                   video_kwargs={"n_objects": SWEEP320_OBJECTS[rate]})
    elif index == 2:
        c = Config("cfg2-scene-labeling-320x240", 2, scene_labeling_net(), 240, 320, 3, 100, 0.02, 0.005,
                   video_kwargs={"n_objects": 3})
    elif index == 3:
        rate = 0.02 if change_rate is None else float(change_rate)
        if rate >= 1.0:
            vk = {"n_objects": 0, "flicker": True}
        else:
            vk = {"n_objects": SWEEP_OBJECTS[rate]}
        c = Config("cfg3-scene-labeling-1280x720-rate%g" % rate, 3, scene_labeling_net(), 720, 1280, 3,
                   200, 0.02, 0.0, video_kwargs=vk)
    elif index == 4:
        c = Config("cfg4-vgg10-640x480-bf16", 4, vgg10_net(), 480, 640, 3, 100, 0.05, 0.01,
                   dtype="bf16", video_kwargs={"n_objects": 5})
    elif index == 5:
        c = Config("cfg5-64-streams-320x240", 5, scene_labeling_net(), 240, 320, 3, 100, 0.02, 0.005,
                   n_streams=64, video_kwargs={"n_objects_fn": _cfg5_count})
    elif index == 6:
        # A strided first layer and other filter sizes (Section 3: a strided convolution drops the unused
        # columns of the image matrix): conv 5x5 / stride 2, conv 3x3, conv 1x1 on 640x480 frames; the
        # sensor noise stays below the threshold, so only the moving objects are recomputed.
        c = Config("cfg6-strided-640x480", 6, strided_net(), 480, 640, 3, 100, 0.02, 0.002,
                   video_kwargs={"n_objects": 5})
    else:
        raise ValueError("config index must be 1..6")
    if height is not None:
        c.height = int(height)
    if width is not None:
        c.width = int(width)
    if n_frames is not None:
        c.n_frames = int(n_frames)
    if sigma is not None:
        c.sigma = float(sigma)
    if n_streams is not None:
        c.n_streams = int(n_streams)
    return c
