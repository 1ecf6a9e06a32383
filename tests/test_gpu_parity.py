"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.
Lists, counts and the stored previous input must be bit-exact; feature maps within
|a-b| <= 1e-5 + 1e-4 |b| (float32)."""
import numpy as np
import pytest

import oracle
import paper_1704_04313_amd as cb
from workloads import (conv, pool, get_config, make_weights, scene_labeling_net, SyntheticVideo)

from gpu_util import (assert_features_close, compare_chained, compare_sequence, oracle_layer_inputs, to_dev)

pytestmark = pytest.mark.gpu


def _video(H, W, C=3, sigma=0.005, n_objects=2, seed=0, **kw):
    return SyntheticVideo(H, W, C, seeds=(seed + 1, seed + 2, seed + 3), sigma=sigma, n_objects=n_objects,
                          size_range=kw.pop("size_range", (4, 10)), speed_range=(1, 3), **kw)


# ------------------------------------------------------------------ config 1, as written
def test_config1_every_frame():
    cfg = get_config(1)
    v = cfg.video()
    frames = [v.frame(t) for t in range(cfg.n_frames)]
    stats = compare_sequence(cfg.layers, cfg.weights(), frames, cfg.tau, label="cfg1")
    assert stats[0] == (4096, 4096)
    assert all(80 <= c < 400 for c, _ in stats[1:])      # motion (80) + noise flags


def test_config1_noise_free_counts():
    cfg = get_config(1, sigma=0.0)
    v = cfg.video()
    frames = [v.frame(t) for t in range(cfg.n_frames)]
    stats = compare_sequence(cfg.layers, cfg.weights(), frames, cfg.tau, label="cfg1-clean")
    assert stats[-1] == (80, 224)


@pytest.mark.parametrize("hold", [False, True])
def test_config1_reference_modes(hold):
    cfg = get_config(1)
    v = cfg.video()
    frames = [v.frame(t) for t in range(6)]
    compare_sequence(cfg.layers, cfg.weights(), frames, cfg.tau, hold=hold, label="cfg1-hold%d" % hold)


# ------------------------------------------------------------------ per-layer, teacher-forced
@pytest.fixture(scope="module")
def scene_inputs():
    """Oracle layer inputs of the scene-labeling network on a reduced-size replica of the
    320x240 workload (same recipe, 96x80, 5 frames): several tiles plus ragged tails."""
    layers = scene_labeling_net()
    params = make_weights(layers, 2001)
    v = _video(80, 96, sigma=0.005, n_objects=3, seed=40)
    frames = [v.frame(t) for t in range(5)]
    return layers, params, frames, oracle_layer_inputs(layers, params, frames, 0.02)


@pytest.mark.parametrize("l", [0, 2, 4, 5, 6])
def test_scene_network_layer_teacher_forced(scene_inputs, l):
    layers, params, frames, rec = scene_inputs
    sub = [layers[l]]
    subp = [params[l]]
    if l + 1 < len(layers) and layers[l + 1].kind == "pool":
        sub.append(layers[l + 1])
        subp.append(None)
    compare_sequence(sub, subp, rec[l], 0.02, label="scene L%d" % l)


@pytest.mark.parametrize("l,tau", [(2, 0.3), (4, 1.0)])
def test_scene_network_layer_paper_style_thresholds(scene_inputs, l, tau):
    """Thresholds growing with depth (Section 4.3 selects 0.04, 0.3, 1.0) make deeper layers sparse."""
    layers, params, frames, rec = scene_inputs
    sub, subp = [layers[l]], [params[l]]
    if layers[l + 1].kind == "pool":
        sub.append(layers[l + 1])
        subp.append(None)
    stats = compare_sequence(sub, subp, rec[l], tau, label="scene L%d tau %g" % (l, tau))
    assert stats[-1][1] < stats[0][1]


# ------------------------------------------------------------------ random geometry
CASES = [
    # C, M, kh, kw, stride, pad, H, W, pool
    (3, 16, 7, 7, 1, 3, 37, 45, True),
    (5, 7, 3, 3, 1, 1, 19, 23, False),
    (8, 33, 1, 1, 1, 0, 30, 34, True),
    (4, 20, 5, 3, 2, 1, 33, 40, False),
    (6, 130, 2, 2, 1, 0, 21, 18, False),
    (3, 8, 4, 4, 2, 2, 26, 30, False),
    (16, 64, 3, 3, 3, 0, 31, 29, False),
    (1, 1, 3, 3, 1, 2, 8, 9, False),
    (12, 70, 3, 5, 1, 2, 17, 64, True),
    (2, 6, 9, 16, 1, 7, 20, 40, False),
    (3, 5, 6, 4, 1, 2, 23, 31, True),
    # more than 64 output channels (direct-to-LDS producers), with inputs whose K slices lie inside one
    # filter tap (32 and 64 channels) and one whose slices straddle taps (40 channels)
    (32, 130, 3, 3, 2, 1, 21, 26, False),
    (64, 96, 5, 3, 1, 2, 18, 22, True),
    (40, 100, 3, 3, 1, 1, 15, 17, False),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("hold", [False, True])
@pytest.mark.parametrize("lists", [False, True])
def test_random_geometry(case, hold, lists):
    C, M, kh, kw, s, p, H, W, with_pool = case
    L = conv(C, M, kh, relu=True, stride=s, pad=p)
    L = type(L)("conv", C, M, kh, kw, s, p, True)
    layers = [L]
    Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    if with_pool and Ho % 2 == 0 and Wo % 2 == 0:
        layers.append(pool())
    params = make_weights(layers, 7 + C + M)
    v = _video(H, W, C, sigma=0.004, n_objects=2, seed=C * 100 + M)
    frames = [v.frame(t) for t in range(4)]
    # lists: dilation and index extraction as kernels of their own instead of inside the multiplication
    compare_sequence(layers, params, frames, 0.015, hold=hold, label=str(case), lists_every_frame=lists)


# ------------------------------------------------------------------ degenerate inputs
def test_unchanged_input_triggers_nothing_and_keeps_maps():
    layers = [conv(3, 16, 7), pool()]
    params = make_weights(layers, 3)
    f = _video(32, 32).frame(0)
    compare_sequence(layers, params, [f, f, f], 0.0, label="static")
    net = cb.CBInfer(layers, params, f.shape, 0.0)
    a = net.process_frame(to_dev(f)).cpu().numpy()
    b = net.process_frame(to_dev(f)).cpu().numpy()
    assert net.layer_counts(0) == (0, 0) and net.layer_counts(1) == (-1, 0)
    np.testing.assert_array_equal(a, b)
    net.destroy()


def test_everything_changed_is_dense():
    layers = [conv(3, 16, 7), pool()]
    params = make_weights(layers, 4)
    v = _video(40, 36, n_objects=0, flicker=True)
    stats = compare_sequence(layers, params, [v.frame(t) for t in range(3)], 0.02, label="flicker")
    assert stats[1] == (40 * 36, 40 * 36)


@pytest.mark.parametrize("pos,count", [((0, 0), 16), ((0, 17), 28), ((15, 16), 49), ((30, 33), 16)])
def test_single_pixel_change(pos, count):
    layers = [conv(1, 4, 7, relu=False)]
    params = make_weights(layers, 5)
    a = np.zeros((1, 31, 34), np.float32)
    b = a.copy()
    b[0, pos[0], pos[1]] = 1.0
    stats = compare_sequence(layers, params, [a, b], 0.5, label="pixel %s" % (pos,))
    assert stats[1] == (1, count)


def test_threshold_knife_edge_is_strict():
    layers = [conv(1, 1, 1, relu=False)]
    params = make_weights(layers, 6)
    a = np.zeros((1, 4, 70), np.float32)
    b = a.copy()
    b[0, 0, 0] = 0.5                                              # == tau: not flagged
    b[0, 1, 65] = np.nextafter(np.float32(0.5), np.float32(1))    # just above: flagged
    b[0, 2, 3] = np.nan                                           # NaN difference: not flagged
    net = cb.CBInfer(layers, params, a.shape, 0.5)
    net.process_frame(to_dev(a))
    net.process_frame(to_dev(b))
    np.testing.assert_array_equal(net.read_list(0, cb.LIST_CHANGED), [70 + 65])
    net.destroy()


# ------------------------------------------------------------------ whole network
def test_threshold_zero_equals_dense_mode_bit_for_bit():
    """Section 3.3: a threshold of zero reproduces the non-change-based result.  With noise on every
    pixel everything is recomputed in every frame, the change-based and the dense schedule then run
    the same kernels over the same positions, and the match is exact."""
    layers = scene_labeling_net()
    params = make_weights(layers, 8)
    v = _video(48, 64, sigma=0.01, seed=9)
    cbn = cb.CBInfer(layers, params, (3, 48, 64), 0.0)
    dn = cb.CBInfer(layers, params, (3, 48, 64), 0.0)
    dn.set_mode(True)
    for t in range(4):
        f = to_dev(v.frame(t))
        a = cbn.process_frame(f).cpu().numpy()
        b = dn.process_frame(f).cpu().numpy()
        np.testing.assert_array_equal(a, b)
        assert_features_close(b[0], oracle.dense_forward(layers, params, v.frame(t))[-1], "dense frame %d" % t)
    cbn.destroy()
    dn.destroy()


def test_scene_network_end_to_end_reduced():
    """Whole network, change-based, against the oracle, every layer: the first layer's lists exact,
    deeper lists different only on the threshold's knife edge, and every value that both sides
    computed from equivalent data within the float32 tolerance (gpu_util.compare_chained)."""
    layers = scene_labeling_net()
    params = make_weights(layers, 2001)
    v = _video(80, 96, sigma=0.005, n_objects=3, seed=40)
    n_diff, tainted = compare_chained(layers, params, [v.frame(t) for t in range(6)], 0.02, label="scene 96x80")
    assert tainted <= 0.02


def test_threshold_zero_noise_free_video_matches_dense_mode_within_tolerance():
    """Threshold zero on a noise-free video: most outputs are retained from earlier frames, in which
    the multiplication split its sums differently (the split along K follows the number of
    positions), so the match with dense mode is to rounding, not to the bit; the oracle's dense
    inference is held to the same tolerance (Section 3.3: threshold zero reproduces it)."""
    layers = scene_labeling_net()
    params = make_weights(layers, 8)
    v = _video(48, 64, sigma=0.0, seed=9, n_objects=2)
    cbn = cb.CBInfer(layers, params, (3, 48, 64), 0.0)
    dn = cb.CBInfer(layers, params, (3, 48, 64), 0.0)
    dn.set_mode(True)
    retained = False
    for t in range(5):
        f = to_dev(v.frame(t))
        a = cbn.process_frame(f).cpu().numpy()
        b = dn.process_frame(f).cpu().numpy()
        assert_features_close(a[0], b[0], "change-based against dense mode, frame %d" % t)
        assert_features_close(a[0], oracle.dense_forward(layers, params, v.frame(t))[-1], "against O-dense, frame %d" % t)
        if t:
            retained |= cbn.layer_counts(4)[1] < 12 * 16
    assert retained, "every output was recomputed in every frame; the test is too easy"
    cbn.destroy()
    dn.destroy()


def test_reset_and_mode_switch():
    cfg = get_config(1)
    v = cfg.video()
    params = cfg.weights()
    net = cb.CBInfer(cfg.layers, params, (3, 64, 64), cfg.tau)
    net.process_frame(to_dev(v.frame(0)))
    net.process_frame(to_dev(v.frame(1)))
    assert net.layer_counts(0)[0] < 4096
    net.reset()
    out = net.process_frame(to_dev(v.frame(2))).cpu().numpy()[0]
    assert net.layer_counts(0) == (4096, 4096)
    assert_features_close(out, oracle.dense_forward(cfg.layers, params, v.frame(2))[-1], "after reset")
    net.set_mode(True)
    out = net.process_frame(to_dev(v.frame(3))).cpu().numpy()[0]
    assert net.layer_counts(0) == (4096, 4096)
    np.testing.assert_array_equal(net.read_list(0, cb.LIST_UPDATE), np.arange(4096))
    assert_features_close(out, oracle.dense_forward(cfg.layers, params, v.frame(3))[-1], "dense mode")
    net.destroy()


def test_library_owned_workspace_and_profile_counters():
    cfg = get_config(1)
    v = cfg.video()
    net = cb.CBInfer(cfg.layers, cfg.weights(), (3, 64, 64), cfg.tau, caller_workspace=False)
    net.set_profiling(True)
    for t in range(3):
        net.process_frame(to_dev(v.frame(t)))
    ms, n = net.read_profile(0, cb.STEP_NAMES.index("gemm"))
    assert n == 3 and ms > 0
    ms, n = net.read_profile(0, cb.STEP_NAMES.index("detect"))
    assert n == 3 and ms > 0
    net.destroy()


def test_multi_stream_lists_are_concatenated_per_stream():
    layers = [conv(3, 16, 7), pool()]
    params = make_weights(layers, 12)
    S, H, W = 3, 24, 40
    vids = [_video(H, W, seed=100 + s, n_objects=1 + s) for s in range(S)]
    net = cb.CBInfer(layers, params, (3, H, W), 0.02, n_streams=S)
    orcs = [oracle.OracleCBNet(layers, params, 0.02) for _ in range(S)]
    for t in range(4):
        fr = np.stack([vv.frame(t) for vv in vids])
        got = net.process_frame(to_dev(fr)).cpu().numpy()
        want = [o.process_frame(fr[s]) for s, o in enumerate(orcs)]
        cl = np.concatenate([o.trace[0]["C"] + s * H * W for s, o in enumerate(orcs)])
        ul = np.concatenate([o.trace[0]["U"] + s * H * W for s, o in enumerate(orcs)])
        pl = np.concatenate([o.trace[1]["P"] + s * (H // 2) * (W // 2) for s, o in enumerate(orcs)])
        np.testing.assert_array_equal(net.read_list(0, cb.LIST_CHANGED), cl)
        np.testing.assert_array_equal(net.read_list(0, cb.LIST_UPDATE), ul)
        np.testing.assert_array_equal(net.read_list(1, cb.LIST_UPDATE), pl)
        for s in range(S):
            assert_features_close(got[s], want[s], "stream %d frame %d" % (s, t))
    net.destroy()


def test_determinism_two_runs_byte_identical():
    layers = scene_labeling_net()
    params = make_weights(layers, 13)
    v = _video(48, 64, seed=21)
    outs = []
    for _ in range(2):
        net = cb.CBInfer(layers, params, (3, 48, 64), 0.02)
        o = [net.process_frame(to_dev(v.frame(t))).cpu().numpy().copy() for t in range(4)]
        outs.append((o, net.read_list(4, cb.LIST_UPDATE)))
        net.destroy()
    for a, b in zip(outs[0][0], outs[1][0]):
        np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(outs[0][1], outs[1][1])


# ------------------------------------------------------------------ exact arithmetic, whole network
def _integer_video(H, W, C, n_frames, seed):
    """Small-integer frames: static background, one moving block, a few +-1 flickers per frame.
    With small-integer weights every sum is an exactly representable integer in float32 and in
    double alike, so the HIP path and the oracle agree bit for bit at every layer and the lists
    of all layers can be compared exactly (no threshold knife-edges)."""
    r = np.random.default_rng(seed)
    bg = r.integers(0, 4, size=(C, H, W)).astype(np.float32)
    tex = r.integers(0, 4, size=(C, 5, 6)).astype(np.float32)
    frames = []
    for t in range(n_frames):
        f = bg.copy()
        y, x = 3 + t % (H - 8), 2 + (2 * t) % (W - 8)     # wraps around on long videos
        f[:, y:y + 5, x:x + 6] = tex
        for _ in range(6):
            c, yy, xx = r.integers(0, C), r.integers(0, H), r.integers(0, W)
            f[c, yy, xx] += float(r.integers(-1, 2))
        frames.append(f)
    return frames


def _integer_params(layers, seed):
    r = np.random.default_rng(seed)
    params = []
    for L in layers:
        if L.kind != "conv":
            params.append(None)
            continue
        w = r.integers(-1, 2, size=(L.cout, L.cin, L.kh, L.kw)).astype(np.float32)
        b = r.integers(-2, 3, size=L.cout).astype(np.float32)
        params.append((w, b))
    return params


@pytest.mark.parametrize("hold", [False, True])
@pytest.mark.parametrize("lists", [False, True])
def test_integer_network_every_layer_bit_exact(hold, lists):
    layers = [conv(3, 8, 3), pool(), conv(8, 20, 3), conv(20, 12, 1), pool(), conv(12, 5, 3, relu=False)]
    params = _integer_params(layers, 31)
    H, W = 24, 36
    frames = _integer_video(H, W, 3, 7, 77)
    taus = [0.5, None, 1.5, 2.5, None, 3.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, hold_reference=hold, lists_every_frame=lists)
    orc = oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus], ref_mode=1 if hold else 0)
    sparse_seen = False
    for t, f in enumerate(frames):
        want = orc.process_frame(f)
        got = net.process_frame(to_dev(f)).cpu().numpy()[0]
        for l, L in enumerate(layers):
            what = "layer %d frame %d" % (l, t)
            if L.kind == "conv":
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), orc.trace[l]["C"], err_msg=what)
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["U"], err_msg=what)
                np.testing.assert_array_equal(net.read_map(l, cb.MAP_REFERENCE)[0], orc.ref[l], err_msg=what)
                if t and l >= 2 and 0 < orc.trace[l]["C"].size < orc.trace[l]["x"][0].size:
                    sparse_seen = True
            else:
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["P"], err_msg=what)
            np.testing.assert_array_equal(net.read_map(l, cb.MAP_OUTPUT)[0], orc.out[l], err_msg=what)
        np.testing.assert_array_equal(got, want)
    assert sparse_seen, "the deeper layers never saw a sparse change list; the test is too easy"
    net.destroy()


def test_integer_network_reset_and_dense_switch_keep_lists_exact():
    """Resetting and switching modes in mid-video must leave the fused change bitmaps clean."""
    layers = [conv(3, 8, 3), pool(), conv(8, 16, 3), conv(16, 4, 1, relu=False)]
    params = _integer_params(layers, 32)
    frames = _integer_video(20, 28, 3, 8, 78)
    taus = [0.5, None, 1.5, 2.5]
    net = cb.CBInfer(layers, params, (3, 20, 28), taus)
    orc = oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus])
    for t, f in enumerate(frames):
        if t == 3:
            net.reset()
            orc.reset()
        if t == 5:
            net.set_mode(True)
            net.process_frame(to_dev(frames[0]))
            net.set_mode(False)
            orc.reset()
        want = orc.process_frame(f)
        got = net.process_frame(to_dev(f)).cpu().numpy()[0]
        for l in (0, 2, 3):
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), orc.trace[l]["C"],
                                          err_msg="layer %d frame %d" % (l, t))
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["U"])
        np.testing.assert_array_equal(got, want)
    net.destroy()


# ------------------------------------------------------------------ worst-case change propagation
@pytest.mark.parametrize("prop,hold", [((2,), False), ((3,), False), ((2, 3, 5), False), ((5,), False),
                                       ((2, 3, 5), True), ((3,), True)])
def test_integer_network_with_propagating_layers_bit_exact(prop, hold):
    """Layers that run no detection and take the positions recomputed before them as changed
    (Section 4.7), behind a pooling layer, behind a convolution, behind a 1x1 layer."""
    layers = [conv(3, 8, 3), pool(), conv(8, 20, 3), conv(20, 12, 1), pool(), conv(12, 5, 3, relu=False)]
    params = _integer_params(layers, 31)
    H, W = 24, 36
    frames = _integer_video(H, W, 3, 6, 77)
    taus = [0.5, None, 1.5, 2.5, None, 3.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, propagate_layers=prop, hold_reference=hold)
    orc = oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus], propagate_layers=prop,
                             ref_mode=1 if hold else 0)
    for t, f in enumerate(frames):
        want = orc.process_frame(f)
        got = net.process_frame(to_dev(f)).cpu().numpy()[0]
        for l, L in enumerate(layers):
            what = "layer %d frame %d" % (l, t)
            if L.kind == "conv":
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), orc.trace[l]["C"], err_msg=what)
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["U"], err_msg=what)
            else:
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["P"], err_msg=what)
            np.testing.assert_array_equal(net.read_map(l, cb.MAP_OUTPUT)[0], orc.out[l], err_msg=what)
        np.testing.assert_array_equal(got, want)
    net.destroy()


def test_scene_network_all_layers_propagating_lists_exact():
    """With propagation in every layer behind the first, no list depends on a floating-point
    comparison of computed values, so all lists of the whole network must match exactly."""
    layers = scene_labeling_net()
    params = make_weights(layers, 2001)
    H, W, tau = 80, 96, 0.02
    v = _video(H, W, sigma=0.005, n_objects=3, seed=40)
    conv_ids = [l for l, L in enumerate(layers) if L.kind == "conv"]
    net = cb.CBInfer(layers, params, (3, H, W), tau, propagate_layers=conv_ids[1:])
    orc = oracle.OracleCBNet(layers, params, tau, propagate_layers=conv_ids[1:])
    for t in range(4):
        f = v.frame(t)
        want = orc.process_frame(f)
        got = net.process_frame(to_dev(f)).cpu().numpy()[0]
        for l in conv_ids:
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), orc.trace[l]["C"])
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["U"])
            assert net.layer_counts(l) == (orc.trace[l]["C"].size, orc.trace[l]["U"].size)
        assert_features_close(got, want, "network output frame %d" % t)
    net.destroy()


# ------------------------------------------------------------------ index extraction inside / outside the consumers
@pytest.mark.parametrize("W", [512, 516])
def test_selection_map_size_boundary(W):
    """Maps of up to 131072 positions are ranked inside the multiplication kernel, larger ones go
    through the extraction kernel: 256 x 512 is the largest of the first kind, 256 x 516 the
    first multiple of four columns of the second.  Both must give the oracle's lists and values."""
    layers = [conv(3, 4, 3), pool()]
    params = make_weights(layers, 17)
    v = _video(256, W, sigma=0.003, n_objects=4, seed=300 + W, size_range=(6, 20))
    frames = [v.frame(t) for t in range(3)]
    stats = compare_sequence(layers, params, frames, 0.02, label="256x%d" % W)
    assert 0 < stats[-1][0] < 256 * W // 4


@pytest.mark.parametrize("C", [1, 2, 3, 5, 6, 7])
@pytest.mark.parametrize("hold", [False, True])
def test_large_frames_stored_without_padding_channels(C, hold):
    """From 2^18 pixels on a float32 frame whose channel count is no multiple of four is stored
    with C values per pixel (the detection pass then moves no padding); the gathers read 16 bytes
    from any 4-byte word.  Frame size chosen so that the last wave and the last float4 of the map
    are ragged."""
    H, W = 509, 517
    layers = [conv(C, 4, 3)]
    params = make_weights(layers, 60 + C)
    v = _video(H, W, C, sigma=0.003, n_objects=5, seed=700 + C, size_range=(10, 30))
    frames = [v.frame(t) for t in range(3)]
    stats = compare_sequence(layers, params, frames, 0.02, hold=hold, label="C=%d" % C)
    assert 0 < stats[-1][0] < H * W // 4


@pytest.mark.parametrize("lists", [False, True])
def test_integer_network_three_streams_every_layer_bit_exact(lists):
    """Three streams through a network with pooling and a 5x5 layer, stream sizes that are no
    multiple of 64 positions (bitmap words straddle the streams); with `lists` the dilation and
    extraction kernels see byte change maps, pooled maps and stream boundaries together."""
    layers = [conv(3, 6, 3), pool(), conv(6, 9, 5), pool(), conv(9, 4, 3, relu=False)]
    params = _integer_params(layers, 33)
    S, H, W = 3, 20, 28
    vids = [_integer_video(H, W, 3, 5, 200 + s) for s in range(S)]
    taus = [0.5, None, 1.5, None, 2.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, n_streams=S, lists_every_frame=lists)
    orcs = [oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus]) for _ in range(S)]
    for t in range(5):
        fr = np.stack([vids[s][t] for s in range(S)])
        want = np.stack([orcs[s].process_frame(fr[s]) for s in range(S)])
        got = net.process_frame(to_dev(fr)).cpu().numpy()
        for l, L in enumerate(layers):
            what = "layer %d frame %d" % (l, t)
            size = orcs[0].out[l].shape[1] * orcs[0].out[l].shape[2]
            if L.kind == "conv":
                n_in = orcs[0].trace[l]["x"][0].size
                c = np.concatenate([orcs[s].trace[l]["C"] + s * n_in for s in range(S)])
                u = np.concatenate([orcs[s].trace[l]["U"] + s * size for s in range(S)])
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), c, err_msg=what)
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), u, err_msg=what)
            else:
                pl = np.concatenate([orcs[s].trace[l]["P"] + s * size for s in range(S)])
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), pl, err_msg=what)
            m = net.read_map(l, cb.MAP_OUTPUT)
            for s in range(S):
                np.testing.assert_array_equal(m[s], orcs[s].out[l], err_msg=what)
        np.testing.assert_array_equal(got, want)
    net.destroy()


def _random_integer_case(seed, n_frames=5):
    """A random stack of 2-5 convolution layers (1x1 to 7x7, pooling in between, one to three
    streams, either reference mode, either list path, some layers propagating) with integer
    weights and integer videos."""
    r = np.random.default_rng(4242 + seed)
    H, W = int(r.integers(12, 40)) * 2, int(r.integers(12, 50)) * 2
    C, S = int(r.integers(1, 6)), int(r.choice([1, 1, 2, 3]))
    layers, c, h, w = [], C, H, W
    depth = int(r.integers(2, 6))
    for d in range(depth):
        k, m = int(r.choice([1, 1, 3, 3, 5, 7])), int(r.choice([2, 4, 5, 8, 12, 20]))
        layers.append(conv(c, m, k, relu=d < depth - 1))
        c = m
        if r.integers(0, 3) == 0 and h % 2 == 0 and w % 2 == 0 and h >= 8 and w >= 8 and d < depth - 1:
            layers.append(pool())
            h, w = h // 2, w // 2
    hold, lists = bool(r.integers(0, 2)), bool(r.integers(0, 2))
    prop = [l for l, L in enumerate(layers) if L.kind == "conv" and l > 0 and r.integers(0, 5) == 0 and not hold]
    params = _integer_params(layers, int(r.integers(0, 1000)))
    taus = [float(r.choice([0.5, 1.5, 2.5])) if L.kind == "conv" else None for L in layers]
    vids = [_integer_video(H, W, C, n_frames, 300 + seed * 7 + s) for s in range(S)]
    return dict(layers=layers, params=params, taus=taus, vids=vids, H=H, W=W, C=C, S=S, hold=hold, lists=lists, prop=prop)


def _compare_all_layers(net, orcs, layers, S, what):
    for l, L in enumerate(layers):
        size = orcs[0].out[l].shape[1] * orcs[0].out[l].shape[2]
        if L.kind == "conv":
            n_in = orcs[0].trace[l]["x"][0].size
            cl = np.concatenate([orcs[s].trace[l]["C"] + s * n_in for s in range(S)])
            ul = np.concatenate([orcs[s].trace[l]["U"] + s * size for s in range(S)])
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), cl, err_msg="%s layer %d" % (what, l))
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), ul, err_msg="%s layer %d" % (what, l))
        else:
            pl = np.concatenate([orcs[s].trace[l]["P"] + s * size for s in range(S)])
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), pl, err_msg="%s layer %d" % (what, l))
        m = net.read_map(l, cb.MAP_OUTPUT)
        for s in range(S):
            np.testing.assert_array_equal(m[s], orcs[s].out[l], err_msg="%s layer %d" % (what, l))


@pytest.mark.parametrize("seed", range(24))
def test_random_integer_networks_bit_exact(seed):
    """Random networks with integer weights: every layer's lists and maps must match the oracle
    bit for bit on every frame."""
    k = _random_integer_case(seed)
    layers, S = k["layers"], k["S"]
    net = cb.CBInfer(layers, k["params"], (k["C"], k["H"], k["W"]), k["taus"], n_streams=S, hold_reference=k["hold"],
                     lists_every_frame=k["lists"], propagate_layers=k["prop"])
    orcs = [oracle.OracleCBNet(layers, k["params"], [0.0 if t is None else t for t in k["taus"]],
                               ref_mode=1 if k["hold"] else 0, propagate_layers=k["prop"]) for _ in range(S)]
    for t in range(5):
        fr = np.stack([k["vids"][s][t] for s in range(S)])
        want = np.stack([orcs[s].process_frame(fr[s]) for s in range(S)])
        got = net.process_frame(to_dev(fr)).cpu().numpy()
        _compare_all_layers(net, orcs, layers, S, "seed %d frame %d" % (seed, t))
        np.testing.assert_array_equal(got, want)
    net.destroy()


@pytest.mark.parametrize("seed", range(12))
def test_frames_in_flight_bit_exact(seed):
    """Throughput mode (consecutive frames overlap on two streams of the library): 16 frames are
    enqueued back to back without waiting for any of them, each with an output buffer of its own;
    every frame's output, and the lists and maps left by the last one, must equal the oracle's bit
    for bit -- each frame has to see exactly the state the frame before it left."""
    import torch
    T = 16
    k = _random_integer_case(seed, n_frames=T)
    layers, S = k["layers"], k["S"]
    net = cb.CBInfer(layers, k["params"], (k["C"], k["H"], k["W"]), k["taus"], n_streams=S, hold_reference=k["hold"],
                     lists_every_frame=k["lists"], propagate_layers=k["prop"], pipeline_frames=True)
    orcs = [oracle.OracleCBNet(layers, k["params"], [0.0 if t is None else t for t in k["taus"]],
                               ref_mode=1 if k["hold"] else 0, propagate_layers=k["prop"]) for _ in range(S)]
    frames = [to_dev(np.stack([k["vids"][s][t] for s in range(S)])) for t in range(T)]
    outs = [torch.empty(net.out_shape, dtype=torch.float32, device="cuda") for _ in range(T)]
    torch.cuda.synchronize()
    for t in range(T):
        net.process_frame(frames[t], outs[t])
    net.flush()
    torch.cuda.synchronize()
    for t in range(T):
        want = np.stack([orcs[s].process_frame(k["vids"][s][t]) for s in range(S)])
        np.testing.assert_array_equal(outs[t].cpu().numpy(), want, err_msg="seed %d frame %d" % (seed, t))
    _compare_all_layers(net, orcs, layers, S, "seed %d after the last frame" % seed)
    # and onwards after a query (which waits for everything in flight), a reset and a mode switch
    net.reset()
    for s in range(S):
        orcs[s].reset()
    for t in (3, 4, 5):
        fr = np.stack([k["vids"][s][t] for s in range(S)])
        want = np.stack([orcs[s].process_frame(fr[s]) for s in range(S)])
        got = net.process_frame(to_dev(fr))
        net.flush()
        np.testing.assert_array_equal(got.cpu().numpy(), want, err_msg="seed %d frame %d after reset" % (seed, t))
    net.destroy()


def test_frames_in_flight_scene_network_matches_ordinary_mode():
    """The scene-labeling network on noisy video, 24 frames in flight against the same frames one
    at a time: same kernels, same state per frame, so every output must be identical."""
    import torch
    layers = scene_labeling_net()
    params = make_weights(layers, 77)
    v = _video(96, 128, sigma=0.005, n_objects=3, seed=70)
    frames = [to_dev(v.frame(t)) for t in range(24)]
    a = cb.CBInfer(layers, params, (3, 96, 128), 0.02)
    ref = [a.process_frame(f).cpu().numpy().copy() for f in frames]
    a.destroy()
    b = cb.CBInfer(layers, params, (3, 96, 128), 0.02, pipeline_frames=True)
    outs = [torch.empty(b.out_shape, dtype=torch.float32, device="cuda") for _ in frames]
    for f, o in zip(frames, outs):
        b.process_frame(f, o)
    b.flush()
    torch.cuda.synchronize()
    for t, (o, r) in enumerate(zip(outs, ref)):
        np.testing.assert_array_equal(o.cpu().numpy(), r, err_msg="frame %d" % t)
    b.destroy()


@pytest.mark.parametrize("bf16", [False, True])
def test_frames_in_flight_deep_network_matches_ordinary_mode(bf16):
    """A network of thirteen operations (the VGG-style recipe at 64x80), where only every fourth
    operation waits for the previous frame: 20 frames in flight against the same frames one at a
    time, every output identical."""
    import torch
    cfg = get_config(4, height=64, width=80, n_frames=20)
    params = cfg.weights()
    v = cfg.video()
    frames = [to_dev(v.frame(t)) for t in range(cfg.n_frames)]
    dt = cb.BF16 if bf16 else cb.F32
    assert len(cfg.layers) >= 12
    a = cb.CBInfer(cfg.layers, params, (3, 64, 80), cfg.tau, dtype=dt)
    ref = [a.process_frame(f).cpu().numpy().copy() for f in frames]
    a.destroy()
    b = cb.CBInfer(cfg.layers, params, (3, 64, 80), cfg.tau, dtype=dt, pipeline_frames=True)
    outs = [torch.empty(b.out_shape, dtype=torch.float32, device="cuda") for _ in frames]
    for f, o in zip(frames, outs):
        b.process_frame(f, o)
    b.flush()
    torch.cuda.synchronize()
    for t, (o, r) in enumerate(zip(outs, ref)):
        np.testing.assert_array_equal(o.cpu().numpy(), r, err_msg="frame %d" % t)
    b.destroy()


def test_large_multi_stream_frames_without_padding_channels():
    """Two streams whose frames together pass 2^18 pixels (stored with three values per pixel), an
    odd number of pixels per stream: waves and float4 of the stored map straddle the stream boundary."""
    layers = [conv(3, 5, 3)]
    params = make_weights(layers, 71)
    S, H, W = 2, 363, 365
    vids = [_video(H, W, seed=800 + s, n_objects=3, sigma=0.003, size_range=(8, 24)) for s in range(S)]
    net = cb.CBInfer(layers, params, (3, H, W), 0.02, n_streams=S)
    orcs = [oracle.OracleCBNet(layers, params, 0.02) for _ in range(S)]
    for t in range(3):
        fr = np.stack([vv.frame(t) for vv in vids])
        got = net.process_frame(to_dev(fr)).cpu().numpy()
        want = [o.process_frame(fr[s]) for s, o in enumerate(orcs)]
        cl = np.concatenate([o.trace[0]["C"] + s * H * W for s, o in enumerate(orcs)])
        ul = np.concatenate([o.trace[0]["U"] + s * H * W for s, o in enumerate(orcs)])
        np.testing.assert_array_equal(net.read_list(0, cb.LIST_CHANGED), cl)
        np.testing.assert_array_equal(net.read_list(0, cb.LIST_UPDATE), ul)
        ref = net.read_map(0, cb.MAP_REFERENCE)
        for s in range(S):
            np.testing.assert_array_equal(ref[s], orcs[s].ref[0])
            assert_features_close(got[s], want[s], "stream %d frame %d" % (s, t))
    net.destroy()


@pytest.mark.parametrize("case", ["f32", "bf16", "two_streams", "wide"])
def test_trailing_1x1_layers_bit_exact(case):
    """Two 1x1 layers at the end of a network (the classification layers of the paper's network
    are of this kind): each finds its changes while the layer before it writes its output.
    Integer weights: lists and maps of all layers bit for bit, over several frames, one and two
    streams, both storage types, then once more in dense mode."""
    layers = [conv(3, 8, 3), conv(8, 64 if case == "wide" else 6, 1), conv(64 if case == "wide" else 6, 4, 1, relu=False)]
    params = _integer_params(layers, 51)
    H, W = 24, 36
    S = 2 if case == "two_streams" else 1
    bf16 = case == "bf16"
    frames = [_integer_video(H, W, 3, 6, 90 + s) for s in range(S)]
    taus = [0.5, 1.5, 2.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, n_streams=S, dtype=cb.BF16 if bf16 else cb.F32)
    orcs = [oracle.OracleCBNet(layers, params, taus, bf16=bf16) for _ in range(S)]
    No = H * W
    sparse_seen = False
    for t in range(6):
        want = np.stack([orcs[s].process_frame(frames[s][t]) for s in range(S)])
        x = np.stack([frames[s][t] for s in range(S)])
        got = net.process_frame(to_dev(x)).cpu().numpy()
        for l in range(3):
            what = "%s layer %d frame %d" % (case, l, t)
            c_want = np.concatenate([orcs[s].trace[l]["C"] + s * No for s in range(S)])
            u_want = np.concatenate([orcs[s].trace[l]["U"] + s * No for s in range(S)])
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), c_want, err_msg=what)
            np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), u_want, err_msg=what)
            m = net.read_map(l, cb.MAP_OUTPUT)
            for s in range(S):
                np.testing.assert_array_equal(m[s], orcs[s].out[l], err_msg=what)
            if t and l == 2 and 0 < u_want.size < S * No:
                sparse_seen = True
        np.testing.assert_array_equal(got, want)
    assert sparse_seen
    net.set_mode(True)
    dense = net.process_frame(to_dev(np.stack([frames[s][2] for s in range(S)])))
    want = np.stack([oracle.dense_forward(layers, params, frames[s][2], bf16=bf16)[-1] for s in range(S)])
    np.testing.assert_array_equal(dense.cpu().numpy(), want)
    net.destroy()


@pytest.mark.parametrize("hold", [False, True])
def test_integer_network_large_maps_lists_exact(hold):
    """Maps beyond 131072 positions at every layer (dilation a word at a time from bit maps and
    from byte maps, with and without pooling behind, group counts handed to the extraction):
    integer weights make every layer's lists and maps comparable bit for bit."""
    layers = [conv(3, 4, 3), conv(4, 4, 5), pool(), conv(4, 4, 7), conv(4, 3, 1, relu=False)]
    params = _integer_params(layers, 41)
    H, W = 528, 1036   # 547008 positions, 8547 words: not a multiple of the extraction's group size
    frames = _integer_video(H, W, 3, 3, 78)
    taus = [0.5, 1.5, None, 2.5, 3.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, hold_reference=hold)
    orc = oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus], ref_mode=1 if hold else 0)
    for t, f in enumerate(frames):
        want = orc.process_frame(f)
        got = net.process_frame(to_dev(f)).cpu().numpy()[0]
        for l, L in enumerate(layers):
            what = "layer %d frame %d" % (l, t)
            if L.kind == "conv":
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), orc.trace[l]["C"], err_msg=what)
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["U"], err_msg=what)
            else:
                np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), orc.trace[l]["P"], err_msg=what)
            np.testing.assert_array_equal(net.read_map(l, cb.MAP_OUTPUT)[0], orc.out[l], err_msg=what)
        np.testing.assert_array_equal(got, want)
        if t:
            assert 0 < orc.trace[3]["U"].size < (H // 2) * (W // 2) // 10
    net.destroy()


@pytest.mark.parametrize("hold", [False, True])
def test_sparse_changes_far_apart(hold):
    """A handful of single changed pixels spread over a map of many bitmap words: the wanted ranks
    of a tile then lie in words that are far apart."""
    layers = [conv(2, 5, 3, relu=False)]
    params = make_weights(layers, 23)
    r = np.random.default_rng(5)
    base = r.random((2, 96, 200)).astype(np.float32)
    frames = [base]
    for t in range(1, 5):
        f = frames[-1].copy()
        for _ in range(t):      # t isolated pixels
            y, x = int(r.integers(0, 96)), int(r.integers(0, 200))
            f[:, y, x] += 0.5
        frames.append(f)
    stats = compare_sequence(layers, params, frames, 0.1, hold=hold, label="sparse")
    assert [c for c, _ in stats[1:]] == [1, 2, 3, 4]
