"""GPU parity at the benchmark's full sizes (same launch configuration bench.py times).
Config 2 (320x240) is small enough for a complete teacher-forced comparison of every layer on a
few frames; the 1280x720 and the 64-stream shapes are checked with exact lists on the full maps
and feature values on sampled positions that the oracle computes one by one."""
import numpy as np
import pytest

import paper_1704_04313_amd as cb
from workloads import conv, get_config, make_weights

from gpu_util import compare_sampled, compare_sequence, oracle_layer_inputs, to_dev
import oracle

pytestmark = pytest.mark.gpu


def test_config2_full_size_every_layer_teacher_forced():
    cfg = get_config(2)
    params = cfg.weights()
    v = cfg.video()
    frames = [v.frame(t) for t in range(3)]
    rec = oracle_layer_inputs(cfg.layers, params, frames, cfg.tau)
    for l, L in enumerate(cfg.layers):
        if L.kind != "conv":
            continue
        sub, subp = [L], [params[l]]
        if l + 1 < len(cfg.layers) and cfg.layers[l + 1].kind == "pool":
            sub.append(cfg.layers[l + 1])
            subp.append(None)
        stats = compare_sequence(sub, subp, rec[l], cfg.tau, label="cfg2 L%d" % l)
        assert stats[0][1] == rec[l][0].shape[1] * rec[l][0].shape[2]


def _patched_sequence(C, H, W, n_frames, seed, scale=1.0, patches=12):
    """Random map, then copies with a few rectangular patches redrawn per frame (seeded; stands in
    for the layer inputs of the 1280x720 workload, whose complete oracle run would take minutes)."""
    r = np.random.default_rng(seed)
    x = (r.random((C, H, W), dtype=np.float32) * scale).astype(np.float32)
    seq = [x]
    for t in range(1, n_frames):
        y = seq[-1].copy()
        for _ in range(patches):
            h, w = int(r.integers(3, 20)), int(r.integers(3, 30))
            y0, x0 = int(r.integers(0, H - h)), int(r.integers(0, W - w))
            y[:, y0:y0 + h, x0:x0 + w] = r.random((C, h, w), dtype=np.float32) * scale
        seq.append(y)
    return seq


@pytest.mark.parametrize("shape", [
    # C, M, k, H, W  -- the layer shapes of the scene-labeling network at 1280x720
    (3, 16, 7, 720, 1280),
    (16, 64, 7, 360, 640),
    (64, 256, 7, 180, 320),
    (256, 64, 1, 180, 320),
    (64, 8, 1, 180, 320),
])
def test_config3_layer_shapes_full_size_sampled(shape):
    C, M, k, H, W = shape
    L = conv(C, M, k)
    params = make_weights([L], 3000 + C)[0]
    frames = _patched_sequence(C, H, W, 3, seed=C * 7 + k)
    compare_sampled(L, params, frames, 0.02, label="720p layer %s" % (shape,))


def test_config3_first_layer_full_size_real_video():
    cfg = get_config(3, change_rate=0.02)
    v = cfg.video()
    frames = [v.frame(t) for t in range(3)]
    compare_sampled(cfg.layers[0], cfg.weights()[0], frames, cfg.tau, label="cfg3 L0")


def test_config5_first_layer_64_streams_sampled():
    cfg = get_config(5)
    vids = [cfg.video(s) for s in range(cfg.n_streams)]
    frames = [np.stack([vv.frame(t) for vv in vids]) for t in range(3)]
    compare_sampled(cfg.layers[0], cfg.weights()[0], frames, cfg.tau, n_streams=cfg.n_streams, n_samples=200,
                    label="cfg5 L0")


@pytest.mark.parametrize("l", [0, 1, 2])
def test_strided_workload_layers_full_size_sampled(l):
    """The strided / mixed-filter-size workload (5x5 stride 2, 3x3, 1x1 on 640x480) layer by layer at
    full size: exact lists on the whole maps, feature values on sampled positions.  The first layer
    sees the real video (its 307200-position change map goes through the word-wise dilation at
    stride 2), the deeper ones patched random maps of their input shape."""
    cfg = get_config(6)
    params = cfg.weights()
    L = cfg.layers[l]
    if l == 0:
        v = cfg.video()
        frames = [v.frame(t) for t in range(3)]
    else:
        frames = _patched_sequence(L.cin, 240, 320, 3, seed=600 + l)
    compare_sampled(L, params[l], frames, cfg.tau, label="strided workload layer %d" % l)


@pytest.mark.parametrize("shape", [
    # C, M, k, H, W, bf16 -- layers whose filter rows are short enough for the kernel in which a wave
    # multiplies 16 positions by itself: 2 and 4 channel tiles of 16, taken together by one wave (many
    # positions) or one per wave (few), in both storage types
    (3, 64, 3, 480, 640, False),
    (3, 32, 3, 480, 640, False),
    (16, 32, 3, 60, 80, False),
    (32, 64, 1, 60, 80, False),
    (128, 16, 1, 120, 160, False),
    (3, 32, 3, 480, 640, True),
    (16, 32, 3, 60, 80, True),
    (64, 64, 1, 240, 320, True),
])
def test_short_reduction_layers_sampled(shape):
    C, M, k, H, W, bf16 = shape
    L = conv(C, M, k)
    params = make_weights([L], 4000 + C + M)[0]
    frames = _patched_sequence(C, H, W, 3, seed=C * 11 + M)
    compare_sampled(L, params, frames, 0.02, label="short reduction %s" % (shape,), bf16=bf16)


def test_config2_dominant_layer_thirty_frames_every_tile_shared():
    """The 64 -> 256 7x7 layer at the benchmark's size (4800 positions: 150 tiles over 256
    workgroups, every tile's sum split along K and added up by whichever workgroup finishes last),
    fed the oracle's inputs of that layer for 30 frames; stops at the first frame that differs."""
    cfg = get_config(2)
    params = cfg.weights()
    v = cfg.video()
    frames = [v.frame(t) for t in range(30)]
    rec = oracle_layer_inputs(cfg.layers, params, frames, cfg.tau)
    stats = compare_sequence([cfg.layers[4]], [params[4]], rec[4], cfg.tau, label="cfg2 L4 x30")
    assert len(stats) == 30 and stats[0][1] == 4800


def test_config3_network_chained_full_size():
    """The 1280x720 network as a whole, three frames of the 2 % sweep video, every layer against the
    oracle (exact first-layer lists, knife-edge rule behind it, values at all positions that both
    sides computed from equivalent data)."""
    from gpu_util import compare_chained
    cfg = get_config(3, change_rate=0.02)
    v = cfg.video()
    compare_chained(cfg.layers, cfg.weights(), [v.frame(t) for t in range(3)], cfg.tau, label="cfg3 720p")


def _sparse_integer_params(layers, seed, nnz, in_max=3.0):
    """Per output channel `nnz` weights of +-1 at random taps, all others zero, small integer biases:
    whatever the order of summation, no partial sum of any layer can leave the integers a float32
    holds exactly (asserted from the layer-by-layer bound nnz * bound + 2)."""
    r = np.random.default_rng(seed)
    params, bound = [], in_max
    for L in layers:
        if L.kind != "conv":
            params.append(None)
            continue
        K = L.cin * L.kh * L.kw
        w = np.zeros((L.cout, K), np.float32)
        for o in range(L.cout):
            w[o, r.choice(K, size=min(nnz, K), replace=False)] = r.choice([-1.0, 1.0], size=min(nnz, K))
        b = r.integers(-2, 3, size=L.cout).astype(np.float32)
        bound = nnz * bound + 2.0
        assert bound < 2 ** 24, "sums of layer %s may not be exact" % (L,)
        params.append((w.reshape(L.cout, L.cin, L.kh, L.kw), b))
    return params


def _integer_frames(H, W, C, n_frames, seed):
    r = np.random.default_rng(seed)
    bg = r.integers(0, 4, size=(C, H, W)).astype(np.float32)
    tex = r.integers(0, 4, size=(C, 12, 17)).astype(np.float32)
    frames = []
    for t in range(n_frames):
        f = bg.copy()
        y, x = 5 + 3 * t, 7 + 2 * t
        f[:, y:y + 12, x:x + 17] = tex
        for _ in range(8):
            c, yy, xx = r.integers(0, C), r.integers(0, H), r.integers(0, W)
            f[c, yy, xx] = float(min(3, max(0, f[c, yy, xx] + r.integers(-1, 2))))
        frames.append(f)
    return frames


def test_config5_all_64_streams_every_layer_bit_exact():
    """The 64-stream workload's shapes (64 x 320x240 through the scene-labeling network, one
    multiplication per layer for all streams) with sparse integer weights and integer frames, so
    that every sum is exact on both sides: the lists of every layer and every stream must equal the
    oracle's bit for bit, and so must the stored maps behind the second convolution and the output."""
    cfg = get_config(5)
    layers = cfg.layers
    params = _sparse_integer_params(layers, 55, nnz=6)
    S, H, W = cfg.n_streams, cfg.height, cfg.width
    vids = [_integer_frames(H, W, 3, 3, 900 + s) for s in range(S)]
    taus = [0.5, None, 1.5, None, 2.5, 2.5, 2.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, n_streams=S)
    orcs = [oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus]) for _ in range(S)]
    try:
        for t in range(3):
            fr = np.stack([vids[s][t] for s in range(S)])
            want = np.stack([orcs[s].process_frame(fr[s]) for s in range(S)])
            got = net.process_frame(to_dev(fr)).cpu().numpy()
            for l, L in enumerate(layers):
                what = "layer %d frame %d" % (l, t)
                size = orcs[0].out[l].shape[1] * orcs[0].out[l].shape[2]
                if L.kind == "conv":
                    n_in = orcs[0].trace[l]["x"][0].size
                    cl = np.concatenate([orcs[s].trace[l]["C"] + s * n_in for s in range(S)])
                    ul = np.concatenate([orcs[s].trace[l]["U"] + s * size for s in range(S)])
                    np.testing.assert_array_equal(net.read_list(l, cb.LIST_CHANGED), cl, err_msg=what)
                    np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), ul, err_msg=what)
                else:
                    pl = np.concatenate([orcs[s].trace[l]["P"] + s * size for s in range(S)])
                    np.testing.assert_array_equal(net.read_list(l, cb.LIST_UPDATE), pl, err_msg=what)
                if l >= 3:
                    m = net.read_map(l, cb.MAP_OUTPUT)
                    for s in range(S):
                        np.testing.assert_array_equal(m[s], orcs[s].out[l], err_msg="%s stream %d" % (what, s))
            np.testing.assert_array_equal(got, want)
            if t:
                assert 0 < orcs[0].trace[4]["U"].size < 4800
    finally:
        net.destroy()


def test_config4_vgg_network_chained_full_size_bit_exact():
    """The VGG-style workload at full size (ten 3x3 layers, 640x480, bfloat16 storage) as a whole
    network: sparse integer weights and integer frames keep every float32 sum exact, so both sides
    round the same sums to bfloat16 and every layer's lists and the output must agree bit for bit."""
    cfg = get_config(4)
    layers = cfg.layers
    params = _sparse_integer_params(layers, 44, nnz=3)
    frames = _integer_frames(cfg.height, cfg.width, 3, 3, 440)
    taus = [0.5 if L.kind == "conv" else None for L in layers]
    net = cb.CBInfer(layers, params, (3, cfg.height, cfg.width), taus, dtype=cb.BF16)
    orc = oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus], bf16=True)
    try:
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
            np.testing.assert_array_equal(got, want)
    finally:
        net.destroy()
