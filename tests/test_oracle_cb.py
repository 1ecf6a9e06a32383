"""Pins for the change-based part of the oracle: values the paper prints, the paper's own
verification rule (threshold zero equals dense inference), brute-force alternatives of the
update set written here, closed forms on the synthetic workload, and error bounds."""
import os

import numpy as np
import pytest

import oracle
from workloads import (conv, pool, get_config, make_weights, scene_labeling_net, SyntheticVideo)


# ---------------------------------------------------------------- change detection
def test_detect_hand_example_strict_and_any_channel():
    tau = np.float32(0.5)
    ref = np.zeros((2, 2, 3), np.float32)
    x = np.zeros((2, 2, 3), np.float32)
    x[0, 0, 0] = 0.5            # exactly tau: strict comparison -> not flagged
    x[1, 0, 1] = -0.75          # negative difference in the second channel only -> flagged
    x[0, 1, 2] = np.nextafter(np.float32(0.5), np.float32(1.0))   # just above -> flagged
    x[1, 1, 0] = np.nan         # NaN compares false -> not flagged
    f = oracle.detect(x, ref, tau)
    np.testing.assert_array_equal(f, [[0, 1, 0], [0, 0, 1]])


def test_detect_uses_float_difference():
    """The difference is formed in float: 1 + 2^-24 - 1 is 0 in float arithmetic."""
    ref = np.full((1, 1, 1), 1.0, np.float32)
    x = np.full((1, 1, 1), 1.0 + 2.0 ** -23, np.float32)
    assert oracle.detect(x, ref, 2.0 ** -24)[0, 0] == 1
    assert oracle.detect(x, ref, 2.0 ** -23)[0, 0] == 0


def test_update_ref_modes():
    ref = np.zeros((2, 1, 3), np.float32)
    x = np.arange(6, dtype=np.float32).reshape(2, 1, 3) + 1
    flag = np.array([[0, 1, 0]], np.uint8)
    r0 = oracle.update_ref(x, ref.copy(), flag, 0)
    np.testing.assert_array_equal(r0, x)
    r1 = oracle.update_ref(x, ref.copy(), flag, 1)
    np.testing.assert_array_equal(r1[:, 0, 1], x[:, 0, 1])
    assert r1[:, 0, 0].sum() == 0 and r1[:, 0, 2].sum() == 0


# ---------------------------------------------------------------- update set
def _scatter_form(flag, kh, kw, s, p, Ho, Wo):
    """Implementation note of Section 3.1: start from an all-zero map; every changed input
    pixel sets the output pixels whose filter support covers it."""
    H, W = flag.shape
    upd = np.zeros((Ho, Wo), np.uint8)
    for yi in range(H):
        for xi in range(W):
            if not flag[yi, xi]:
                continue
            for qy in range(Ho):
                for qx in range(Wo):
                    if 0 <= yi - (qy * s - p) < kh and 0 <= xi - (qx * s - p) < kw:
                        upd[qy, qx] = 1
    return upd


def _closed_ranges(flag, kh, kw, s, p, Ho, Wo):
    """Per changed pixel the affected outputs form the index rectangle
    ceil((yi+p-kh+1)/s) .. floor((yi+p)/s), clipped to the map (same in x)."""
    upd = np.zeros((Ho, Wo), np.uint8)
    for yi, xi in zip(*np.nonzero(flag)):
        y0 = max(0, -((-(yi + p - kh + 1)) // s))
        y1 = min(Ho - 1, (yi + p) // s)
        x0 = max(0, -((-(xi + p - kw + 1)) // s))
        x1 = min(Wo - 1, (xi + p) // s)
        if y0 <= y1 and x0 <= x1:
            upd[y0:y1 + 1, x0:x1 + 1] = 1
    return upd


@pytest.mark.parametrize("seed", range(12))
def test_update_set_three_forms_agree(seed):
    r = np.random.default_rng(seed)
    H, W = int(r.integers(3, 12)), int(r.integers(3, 12))
    kh, kw = int(r.integers(1, 6)), int(r.integers(1, 6))
    kh, kw = min(kh, H), min(kw, W)
    s = int(r.integers(1, 4))
    p = int(r.integers(0, min(kh, kw)))
    flag = (r.random((H, W)) < 0.15).astype(np.uint8)
    Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    got = oracle.update_set(flag, kh, kw, s, p)
    assert got.shape == (Ho, Wo)
    np.testing.assert_array_equal(got, _scatter_form(flag, kh, kw, s, p, Ho, Wo))
    np.testing.assert_array_equal(got, _closed_ranges(flag, kh, kw, s, p, Ho, Wo))


def _golden(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "propagation_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, k, n = line.split()
                vals[name] = (int(k), int(n))
    return vals


def test_printed_propagation_counts(golden_dir):
    g = _golden(golden_dir)
    k, n49 = g["one_pixel_after_first_7x7"]
    flag = np.zeros((31, 33), np.uint8)
    flag[15, 16] = 1
    u1 = oracle.update_set(flag, k, k, 1, 3)
    assert int(u1.sum()) == n49 == 49
    u2 = oracle.update_set(u1, k, k, 1, 3)
    assert int(u2.sum()) == g["one_pixel_after_second_7x7"][1] == 169
    corner = np.zeros((31, 33), np.uint8)
    corner[0, 0] = 1
    assert int(oracle.update_set(corner, k, k, 1, 3).sum()) == g["corner_pixel_7x7_pad3"][1]
    edge = np.zeros((31, 33), np.uint8)
    edge[0, 16] = 1
    assert int(oracle.update_set(edge, k, k, 1, 3).sum()) == g["edge_pixel_7x7_pad3"][1]


def test_extract_is_ascending_and_complete():
    r = np.random.default_rng(0)
    m = (r.random((13, 17)) < 0.3).astype(np.uint8)
    lst = oracle.extract(m)
    assert lst.dtype == np.int32 and lst.size == int(m.sum())
    assert np.all(np.diff(lst) > 0)
    np.testing.assert_array_equal(lst, np.flatnonzero(m.ravel()))


def test_pool_set_is_unique_halved_positions():
    r = np.random.default_rng(2)
    upd = (r.random((10, 14)) < 0.1).astype(np.uint8)
    ps = oracle.pool_set(upd, 2)
    ys, xs = np.nonzero(upd)
    want = np.unique((ys // 2) * 7 + xs // 2)
    np.testing.assert_array_equal(oracle.extract(ps), want)


# ---------------------------------------------------------------- whole layer / network
def _small_net():
    layers = [conv(3, 4, 7), pool(), conv(4, 6, 3), conv(6, 2, 1, relu=False)]
    return layers, make_weights(layers, 123)


def _video(sigma=0.0, n_objects=2, H=20, W=24, **kw):
    return SyntheticVideo(H, W, 3, seeds=(1, 2, 3), sigma=sigma, n_objects=n_objects,
                          size_range=(3, 6), speed_range=(1, 2), **kw)


def test_threshold_zero_equals_dense_bit_for_bit():
    """Section 3.3: a threshold of zero yields results identical to the non-change-based
    implementation."""
    layers, params = _small_net()
    v = _video(sigma=0.01)
    net = oracle.OracleCBNet(layers, params, tau=0.0)
    for t in range(5):
        f = v.frame(t)
        y = net.process_frame(f)
        dense = oracle.dense_forward(layers, params, f)
        for l in range(len(layers)):
            np.testing.assert_array_equal(net.trace[l]["out"], dense[l])
        np.testing.assert_array_equal(y, dense[-1])


def test_threshold_zero_config1():
    cfg = get_config(1)
    params = cfg.weights()
    v = cfg.video()
    net = oracle.OracleCBNet(cfg.layers, params, tau=0.0)
    for t in range(3):
        f = v.frame(t)
        np.testing.assert_array_equal(net.process_frame(f), oracle.dense_forward(cfg.layers, params, f)[-1])


def test_first_frame_is_dense_and_lists_are_identity():
    layers, params = _small_net()
    net = oracle.OracleCBNet(layers, params, tau=0.05)
    f = _video().frame(0)
    net.process_frame(f)
    tr = net.trace[0]
    np.testing.assert_array_equal(tr["C"], np.arange(20 * 24))
    np.testing.assert_array_equal(tr["U"], np.arange(20 * 24))
    np.testing.assert_array_equal(net.trace[1]["P"], np.arange(10 * 12))
    np.testing.assert_array_equal(tr["out"], oracle.dense_forward(layers, params, f)[0])


def test_unchanged_input_triggers_nothing():
    layers, params = _small_net()
    net = oracle.OracleCBNet(layers, params, tau=0.0)
    f = _video().frame(0)
    net.process_frame(f)
    before = [np.array(o, copy=True) for o in net.out]
    net.process_frame(f.copy())
    for l, L in enumerate(layers):
        if L.kind == "conv":
            assert net.trace[l]["C"].size == 0 and net.trace[l]["U"].size == 0
        else:
            assert net.trace[l]["P"].size == 0
        np.testing.assert_array_equal(net.out[l], before[l])


def test_everything_changed_equals_dense():
    """Worst case of Section 3.1: with every pixel changed the reduced multiplication is the
    full-frame convolution."""
    layers, params = _small_net()
    v = _video(n_objects=0, flicker=True)
    net = oracle.OracleCBNet(layers, params, tau=0.02)
    net.process_frame(v.frame(0))
    f = v.frame(1)
    y = net.process_frame(f)
    assert net.trace[0]["U"].size == 20 * 24
    np.testing.assert_array_equal(net.trace[0]["out"], oracle.dense_forward(layers, params, f)[0])


def test_config1_noise_free_closed_form_counts():
    """An 8x8 textured square moved 2 px along x changes the 8x10 union of its old and new
    footprint: 80 pixels = 1.95 % of 64x64, and (away from the border) 14x16 outputs of a
    7x7 layer."""
    cfg = get_config(1, sigma=0.0)
    net = oracle.OracleCBNet(cfg.layers, cfg.weights(), tau=cfg.tau)
    v = cfg.video()
    net.process_frame(v.frame(0))
    for t in range(1, cfg.n_frames):
        net.process_frame(v.frame(t))
        tr = net.trace[0]
        x0 = 10 + 2 * (t - 1)
        want = np.zeros((64, 64), np.uint8)
        want[28:36, x0:x0 + 10] = 1
        # a texture pair closer than tau in all channels is possible but rare: allow subset
        assert np.all(tr["flags"] <= want)
        assert tr["C"].size >= 78
        if tr["C"].size == 80:
            assert tr["U"].size == 14 * 16
            wu = np.zeros((64, 64), np.uint8)
            wu[25:39, x0 - 3:x0 + 13] = 1
            np.testing.assert_array_equal(tr["upd"], wu)
    assert tr["C"].size == 80


def test_list_invariants_and_threshold_monotonicity():
    layers, params = _small_net()
    v = _video(sigma=0.01)
    nets = [oracle.OracleCBNet(layers[:1], params[:1], tau=t) for t in (0.01, 0.03)]
    for t in range(4):
        f = v.frame(t)
        for n in nets:
            n.process_frame(f)
        a, b = nets[0].trace[0], nets[1].trace[0]
        if t:
            assert set(b["C"]).issubset(set(a["C"]))      # same previous input in mode 0
        for tr in (a, b):
            assert np.all(np.diff(tr["C"]) > 0) and np.all(np.diff(tr["U"]) > 0)
            assert tr["C"].size == int(tr["flags"].sum()) and tr["U"].size == int(tr["upd"].sum())
            assert set(tr["C"]).issubset(set(tr["U"]))     # 7x7, stride 1, pad 3: q = p is covered


def _l1(w):
    return np.abs(w.astype(np.float64)).sum(axis=(1, 2, 3))


def test_error_bounds_single_layer_both_modes():
    """Against dense inference on the same input.  Reference held only where flagged:
    every input deviates from the value the stored output was computed from by at most tau,
    so |y_cb - y_dense| <= tau * sum|w_o| ... and never more than 2 tau sum|w_o|.
    Reference = previous frame: a position not recomputed for a frames has inputs that
    drifted by at most a * tau."""
    layers = [conv(3, 5, 7, relu=False)]
    params = make_weights(layers, 9)
    tau = 0.03
    v = _video(sigma=0.01, H=24, W=24)
    l1 = _l1(params[0][0])
    net0 = oracle.OracleCBNet(layers, params, tau=tau, ref_mode=0)
    net1 = oracle.OracleCBNet(layers, params, tau=tau, ref_mode=1)
    age = np.zeros((24, 24), np.int64)
    for t in range(8):
        f = v.frame(t)
        y0, y1 = net0.process_frame(f), net1.process_frame(f)
        d = oracle.dense_forward(layers, params, f)[0]
        upd = net0.trace[0]["upd"].astype(bool)
        age = np.where(upd, 0, age + 1)
        e0 = np.abs(y0.astype(np.float64) - d)
        e1 = np.abs(y1.astype(np.float64) - d)
        assert np.all(e0 <= age[None] * tau * l1[:, None, None] + 1e-5)
        assert np.all(e1 <= 2 * tau * l1[:, None, None] + 1e-5)
        assert np.all(e0[:, upd] <= 1e-6)


def test_drift_ramp_distinguishes_reference_modes():
    """x_t = x_0 + t*delta with delta < tau: never flagged when the reference is the
    previous frame; flagged every ceil(tau/delta)-ish frames when the reference is held."""
    layers = [conv(1, 1, 3, relu=False)]
    params = make_weights(layers, 1)
    x0 = np.full((1, 6, 6), 0.25, np.float32)
    delta, tau = 0.25, 0.6
    n0 = oracle.OracleCBNet(layers, params, tau=tau, ref_mode=0)
    n1 = oracle.OracleCBNet(layers, params, tau=tau, ref_mode=1)
    c0, c1 = [], []
    for t in range(7):
        f = x0 + np.float32(t * delta)
        n0.process_frame(f)
        n1.process_frame(f)
        c0.append(n0.trace[0]["C"].size)
        c1.append(n1.trace[0]["C"].size)
    assert c0 == [36, 0, 0, 0, 0, 0, 0]
    assert c1 == [36, 0, 0, 36, 0, 0, 36]      # |0.75| > 0.6 at t = 3, again 3 frames later


def test_pooling_of_stored_map_is_dense_pooling():
    layers, params = _small_net()
    v = _video(sigma=0.01)
    net = oracle.OracleCBNet(layers, params, tau=0.02)
    for t in range(3):
        net.process_frame(v.frame(t))
        np.testing.assert_array_equal(net.out[1], oracle.maxpool(net.out[0], 2))
        u = net.trace[0]["U"]
        want = np.unique((u // 24 // 2) * 12 + (u % 24) // 2)
        np.testing.assert_array_equal(net.trace[1]["P"], want)


def test_recompute_uses_current_input_everywhere_in_the_support():
    """The reduced X is assembled from the current input, including pixels below threshold."""
    layers = [conv(1, 1, 3, relu=False)]
    w = np.ones((1, 1, 3, 3), np.float32)
    params = [(w, np.zeros(1, np.float32))]
    net = oracle.OracleCBNet(layers, params, tau=0.5)
    a = np.zeros((1, 5, 5), np.float32)
    net.process_frame(a)
    b = a.copy()
    b[0, 2, 2] = 1.0      # flagged
    b[0, 2, 3] = 0.25     # below threshold but inside the support of recomputed outputs
    y = net.process_frame(b)
    assert y[0, 2, 2] == 1.25 and y[0, 2, 4] == 0.0     # (2,4) not recomputed: stale by 0.25
    assert net.trace[0]["U"].size == 9


# ---------------------------------------------------------------- worst-case change propagation
def test_propagation_printed_counts_without_detection(golden_dir):
    """Section 3 / Section 4.7: one changed pixel reaches 7x7 outputs of the first 7x7 layer and,
    if every one of them is taken as changed (no detection in the second layer), 13x13 outputs
    of the second: the counts the paper prints, here produced by the propagating mode itself."""
    vals = {}
    with open(os.path.join(golden_dir, "propagation_counts.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, _, v = line.split()[:3]
                vals[k] = int(v)
    layers = [conv(1, 2, 7, relu=False), conv(2, 1, 7, relu=False)]
    params = make_weights(layers, 5)
    net = oracle.OracleCBNet(layers, params, tau=0.5, propagate_layers=[1])
    a = np.zeros((1, 31, 31), np.float32)
    net.process_frame(a)
    b = a.copy()
    b[0, 15, 15] = 1.0
    net.process_frame(b)
    assert net.trace[0]["U"].size == vals["one_pixel_after_first_7x7"]
    assert net.trace[1]["C"].size == vals["one_pixel_after_first_7x7"]
    assert net.trace[1]["U"].size == vals["one_pixel_after_second_7x7"]


def test_propagation_is_a_superset_of_detection_and_exact_at_threshold_zero():
    """Every position whose input value changed at all was recomputed by the layer before, so the
    propagated set contains the detected set for any threshold; with threshold zero in the first
    layer the propagating network equals per-frame dense inference bit for bit."""
    layers, params = _small_net()
    v = _video(sigma=0.01)
    det = oracle.OracleCBNet(layers, params, tau=0.02)
    conv_ids = [l for l, L in enumerate(layers) if L.kind == "conv"]
    prop = oracle.OracleCBNet(layers, params, tau=0.02, propagate_layers=conv_ids[1:])
    exact = oracle.OracleCBNet(layers, params, tau=0.0, propagate_layers=conv_ids[1:])
    for t in range(5):
        f = v.frame(t)
        det.process_frame(f)
        prop.process_frame(f)
        y = exact.process_frame(f)
        np.testing.assert_array_equal(y, oracle.dense_forward(layers, params, f)[-1])
        # both see the same first-layer input, hence the same first-layer sets
        np.testing.assert_array_equal(det.trace[0]["U"], prop.trace[0]["U"])
        l1 = conv_ids[1]
        assert np.isin(det.trace[l1]["C"], prop.trace[l1]["C"]).all()
        if t:
            assert prop.trace[l1]["C"].size >= det.trace[l1]["C"].size
