"""Network descriptions (shapes only) and seeded He-normal weights.

The layer lists follow the benchmark configurations: a one-layer 7x7 network, the
five-layer scene-labeling style network (7x7 feature extraction layers followed by
1x1 pixel-classification layers; Table 1 of the paper lists the same structure: three
7x7 layers, pooling after the first two, then two classification layers) and a
VGG-style 3x3 stack.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class LayerSpec:
    kind: str            # "conv" | "pool"
    cin: int = 0
    cout: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    relu: bool = False


def conv(cin: int, cout: int, k: int, relu: bool = True, stride: int = 1, pad: int = -1) -> LayerSpec:
    return LayerSpec("conv", cin, cout, k, k, stride, (k - 1) // 2 if pad < 0 else pad, relu)


def pool(k: int = 2) -> LayerSpec:
    return LayerSpec("pool", 0, 0, k, k, k, 0, False)


def single_layer_net() -> List[LayerSpec]:
    return [conv(3, 16, 7, relu=False)]


def scene_labeling_net() -> List[LayerSpec]:
    return [conv(3, 16, 7), pool(), conv(16, 64, 7), pool(), conv(64, 256, 7),
            conv(256, 64, 1), conv(64, 8, 1, relu=False)]


def vgg10_net() -> List[LayerSpec]:
    return [conv(3, 64, 3), conv(64, 64, 3), pool(),
            conv(64, 128, 3), conv(128, 128, 3), pool(),
            conv(128, 256, 3), conv(256, 256, 3), conv(256, 256, 3), pool(),
            conv(256, 512, 3), conv(512, 512, 3), conv(512, 512, 3)]


def strided_net() -> List[LayerSpec]:
    return [conv(3, 32, 5, stride=2), conv(32, 64, 3), conv(64, 8, 1, relu=False)]


def out_shape(layers: Sequence[LayerSpec], c: int, h: int, w: int) -> List[Tuple[int, int, int]]:
    """Shape (C, H, W) after every layer."""
    shapes = []
    for L in layers:
        if L.kind == "conv":
            assert L.cin == c, "channel mismatch"
            h = (h + 2 * L.pad - L.kh) // L.stride + 1
            w = (w + 2 * L.pad - L.kw) // L.stride + 1
            c = L.cout
        else:
            h, w = h // L.kh, w // L.kw
        shapes.append((c, h, w))
    return shapes


def dense_flops(layers: Sequence[LayerSpec], c: int, h: int, w: int) -> List[float]:
    """2*M*K*No per conv layer (0 for pools): the cost of per-frame evaluation."""
    res = []
    for L, (co, ho, wo) in zip(layers, out_shape(layers, c, h, w)):
        res.append(2.0 * L.cout * L.cin * L.kh * L.kw * ho * wo if L.kind == "conv" else 0.0)
    return res


def make_weights(layers: Sequence[LayerSpec], seed: int):
    """He-normal weights N(0, 2/(Cin*kh*kw)) as [M][C][kh][kw] float32 and biases
    uniform in [-0.1, 0.1] as [M] float32, one pair per conv layer (None for pools)."""
    r = np.random.Generator(np.random.PCG64(int(seed)))
    params = []
    for L in layers:
        if L.kind != "conv":
            params.append(None)
            continue
        fan_in = L.cin * L.kh * L.kw
        w = (r.standard_normal((L.cout, L.cin, L.kh, L.kw)) * np.sqrt(2.0 / fan_in)).astype(np.float32)
        b = r.uniform(-0.1, 0.1, size=L.cout).astype(np.float32)
        params.append((w, b))
    return params
