"""Whole-network oracle: dense per-frame evaluation and the change-based evaluation.

TEST INFRASTRUCTURE ONLY.  Composes the C steps in the order Section 3.1 lists them:
change detection -> change-index extraction -> (reduced) matrix generation and
multiplication -> output update, per convolution layer, with the layer state of
Section 3.2 (previous input and previous output per layer).  Pooling is evaluated
densely on the stored map, as in the paper (Table 1 lists it as its own step).
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from . import steps


def dense_forward(layers, params, frame, bf16: bool = False) -> List[np.ndarray]:
    """Per-frame evaluation without any state.  Returns every layer's output."""
    x = np.ascontiguousarray(frame, dtype=np.float32)
    if bf16:
        x = steps.round_bf16(x)
    outs = []
    for L, P in zip(layers, params):
        if L.kind == "conv":
            w, b = P
            if bf16:
                w = steps.round_bf16(w)
            x = steps.conv_dense(x, w, b, L.stride, L.pad, L.relu, bf16)
        else:
            x = steps.maxpool(x, L.kh)
        outs.append(x)
    return outs


class OracleCBNet:
    """Change-based evaluation of a conv/pool sequence on one video stream.

    tau: one threshold for all conv layers, or a sequence with one entry per layer
         (entries at pooling layers are ignored).
    ref_mode: 0 = the stored previous input is the previous frame's input everywhere
              (the x^(t-1) of the detection formula); 1 = it is only refreshed where a
              change was flagged.
    propagate_layers: conv layers (not the first) that run no change detection and take every
              input position recomputed by the layer before them as changed (Section 4.7).
    After process_frame(), self.trace[l] holds, per conv layer: 'x' (its input), 'flags',
    'C' (changed input positions), 'upd' (map), 'U' (outputs recomputed), 'out' (stored
    output after the update); per pooling layer: 'P' (pooled positions touched) and 'out'.
    """

    def __init__(self, layers, params, tau, ref_mode: int = 0, bf16: bool = False,
                 dense_layers: Sequence[int] = (), propagate_layers: Sequence[int] = ()):
        self.layers = list(layers)
        self.params = []
        for L, P in zip(self.layers, params):
            if L.kind == "conv" and bf16:
                self.params.append((steps.round_bf16(P[0]), P[1]))
            else:
                self.params.append(P)
        n = len(self.layers)
        self.tau = [float(tau)] * n if np.isscalar(tau) else [float(t) for t in tau]
        assert len(self.tau) == n
        self.ref_mode = int(ref_mode)
        self.bf16 = bool(bf16)
        self.dense_layers = set(dense_layers)
        self.propagate_layers = set(propagate_layers)
        assert 0 not in self.propagate_layers and not (self.propagate_layers & self.dense_layers)
        self.reset()

    def reset(self):
        self.ref = [None] * len(self.layers)
        self.out = [None] * len(self.layers)
        self.initialised = False
        self.trace = [None] * len(self.layers)

    def process_frame(self, frame) -> np.ndarray:
        x = np.ascontiguousarray(frame, dtype=np.float32)
        if self.bf16:
            x = steps.round_bf16(x)
        prev_upd = None
        for l, (L, P) in enumerate(zip(self.layers, self.params)):
            if L.kind == "conv":
                w, b = P
                Cc, H, W = x.shape
                if not self.initialised or l in self.dense_layers:
                    flags = np.ones((H, W), np.uint8)
                elif l in self.propagate_layers:
                    # worst-case propagation (Section 4.7): no detection; every position the layer
                    # before recomputed (carried through pooling) counts as changed
                    flags = np.array(prev_upd, dtype=np.uint8, copy=True)
                    assert flags.shape == (H, W)
                else:
                    flags = steps.detect(x, self.ref[l], self.tau[l])
                if self.ref[l] is None:
                    self.ref[l] = x.copy()
                else:
                    steps.update_ref(x, self.ref[l], flags, self.ref_mode)
                clist = steps.extract(flags)
                upd = steps.update_set(flags, L.kh, L.kw, L.stride, L.pad)
                ulist = steps.extract(upd)
                if self.out[l] is None:
                    self.out[l] = np.zeros((L.cout,) + upd.shape, np.float32)
                steps.conv_update(x, w, b, ulist, self.out[l], L.stride, L.pad, L.relu, self.bf16)
                self.trace[l] = dict(x=x, flags=flags, C=clist, upd=upd, U=ulist, out=self.out[l])
                prev_upd = upd
                x = self.out[l]
            else:
                self.out[l] = steps.maxpool(x, L.kh)
                pl = None
                if prev_upd is not None:
                    prev_upd = steps.pool_set(prev_upd, L.kh)
                    pl = steps.extract(prev_upd)
                self.trace[l] = dict(x=x, P=pl, out=self.out[l])
                x = self.out[l]
        self.initialised = True
        return x
