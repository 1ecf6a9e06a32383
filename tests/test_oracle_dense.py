"""Pins for the dense parts of the oracle: the convolution layer (Section 3 eq. (1) in its
matrix form) and max-pooling, against textbook routines (torch CPU in float64) and against
a brute-force loop written here."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

SHAPES = [
    # C, H, W, M, kh, kw, stride, pad
    (3, 9, 11, 5, 7, 7, 1, 3),
    (2, 8, 8, 3, 3, 3, 1, 1),
    (4, 10, 7, 6, 1, 1, 1, 0),
    (3, 12, 13, 4, 3, 5, 2, 1),    # non-square kernel, stride 2: catches swapped j/i
    (2, 9, 9, 3, 4, 4, 1, 0),      # even kernel, no padding
    (5, 11, 10, 2, 2, 3, 3, 2),    # pad == kh: padding wider than usual
    (16, 12, 12, 8, 7, 7, 1, 3),
]


@pytest.mark.parametrize("C,H,W,M,kh,kw,s,p", SHAPES)
@pytest.mark.parametrize("relu", [False, True])
def test_conv_matches_torch_fp64(C, H, W, M, kh, kw, s, p, relu):
    if p >= kh or p >= kw:
        p = min(kh, kw) - 1
    r = np.random.default_rng(C * 1000 + H * 10 + kh)
    x = r.standard_normal((C, H, W)).astype(np.float32)
    w = r.standard_normal((M, C, kh, kw)).astype(np.float32)
    b = r.standard_normal(M).astype(np.float32)
    y = oracle.conv_dense(x, w, b, s, p, relu)
    ref = F.conv2d(torch.from_numpy(x).double()[None], torch.from_numpy(w).double(),
                   torch.from_numpy(b).double(), stride=s, padding=p)[0]
    if relu:
        ref = ref.clamp_min(0)
    ref = ref.numpy()
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=1e-6, atol=1e-6)


def test_conv_brute_force_tiny():
    r = np.random.default_rng(5)
    C, H, W, M, kh, kw, s, p = 2, 5, 6, 3, 3, 2, 2, 1
    x = r.standard_normal((C, H, W)).astype(np.float32)
    w = r.standard_normal((M, C, kh, kw)).astype(np.float32)
    b = r.standard_normal(M).astype(np.float32)
    y = oracle.conv_dense(x, w, b, s, p, False)
    Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    xp = np.zeros((C, H + 2 * p, W + 2 * p))
    xp[:, p:p + H, p:p + W] = x
    for o in range(M):
        for qy in range(Ho):
            for qx in range(Wo):
                v = float(b[o]) + float((w[o].astype(np.float64) *
                                         xp[:, qy * s:qy * s + kh, qx * s:qx * s + kw]).sum())
                assert abs(y[o, qy, qx] - v) <= 1e-6 * max(1.0, abs(v))


def test_conv_is_correlation_not_flipped():
    """A single weight at tap (j=0, i=1) must read the input one column to the right of
    the padded origin: y(q) = x(qy - p, qx - p + 1)."""
    x = np.arange(25, dtype=np.float32).reshape(1, 5, 5)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 1] = 1.0
    y = oracle.conv_dense(x, w, None, 1, 1, False)
    assert y[0, 2, 2] == x[0, 1, 2]
    assert y[0, 0, 0] == 0.0          # reads the zero padding above the map
    assert y[0, 1, 0] == x[0, 0, 0]


@pytest.mark.parametrize("C,H,W,k", [(3, 8, 10, 2), (2, 9, 7, 2), (1, 6, 6, 3)])
def test_maxpool_matches_torch(C, H, W, k):
    r = np.random.default_rng(H * W)
    x = r.standard_normal((C, H, W)).astype(np.float32)
    y = oracle.maxpool(x, k)
    ref = F.max_pool2d(torch.from_numpy(x)[None], k, k)[0].numpy()
    np.testing.assert_array_equal(y, ref)


def test_bf16_rounding_matches_torch():
    r = np.random.default_rng(3)
    a = (r.standard_normal(4096) * 10.0 ** r.integers(-6, 6, 4096)).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]   # ties: to even
    got = oracle.round_bf16(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(got, ref)


def test_dense_forward_matches_torch_network():
    from workloads import scene_labeling_net, make_weights
    layers = scene_labeling_net()
    params = make_weights(layers, 11)
    r = np.random.default_rng(1)
    x = r.random((3, 16, 20)).astype(np.float32)
    outs = oracle.dense_forward(layers, params, x)
    t = torch.from_numpy(x).double()[None]
    for L, P, o in zip(layers, params, outs):
        if L.kind == "conv":
            t = F.conv2d(t, torch.from_numpy(P[0]).double(), torch.from_numpy(P[1]).double(),
                         stride=L.stride, padding=L.pad)
            if L.relu:
                t = t.clamp_min(0)
        else:
            t = F.max_pool2d(t, L.kh, L.kh)
        np.testing.assert_allclose(o, t[0].numpy(), rtol=2e-5, atol=2e-6)
