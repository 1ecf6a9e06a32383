"""GPU parity with bfloat16 storage (maps and filter matrices bfloat16, float32 accumulation,
float32 frames, thresholds and bias): the HIP library against the oracle run in its bfloat16
mode (inputs, weights and every stored output rounded to bfloat16, sums in double).

Lists, counts and the stored previous input are bit-exact: both sides compare the same
bfloat16 values.  Stored outputs agree within one bfloat16 step (see gpu_util).  Whole networks
are compared bit for bit with integer-valued data, where rounding to bfloat16 is the same
function of the same exact sum on both sides."""
import numpy as np
import pytest

import oracle
import paper_1704_04313_amd as cb
from workloads import (conv, pool, get_config, make_weights, scene_labeling_net, vgg10_net, SyntheticVideo)

from gpu_util import (assert_features_close, compare_sampled, compare_sequence, oracle_layer_inputs, to_dev)
from test_gpu_parity import CASES, _integer_params, _integer_video, _video

pytestmark = pytest.mark.gpu


def test_config1_bf16_every_frame():
    cfg = get_config(1)
    v = cfg.video()
    frames = [v.frame(t) for t in range(cfg.n_frames)]
    stats = compare_sequence(cfg.layers, cfg.weights(), frames, cfg.tau, label="cfg1 bf16", bf16=True)
    assert stats[0] == (4096, 4096)
    assert all(0 < c < 600 for c, _ in stats[1:])


def _with_pool(layers, params, l):
    sub, subp = [layers[l]], [params[l]]
    if l + 1 < len(layers) and layers[l + 1].kind == "pool":
        sub.append(layers[l + 1])
        subp.append(None)
    return sub, subp


@pytest.fixture(scope="module")
def scene_inputs_bf16():
    layers = scene_labeling_net()
    params = make_weights(layers, 2001)
    v = _video(80, 96, sigma=0.005, n_objects=3, seed=40)
    frames = [v.frame(t) for t in range(5)]
    return layers, params, oracle_layer_inputs(layers, params, frames, 0.02, bf16=True)


@pytest.mark.parametrize("l", [0, 2, 4, 5, 6])
def test_scene_network_layer_teacher_forced_bf16(scene_inputs_bf16, l):
    layers, params, rec = scene_inputs_bf16
    sub, subp = _with_pool(layers, params, l)
    compare_sequence(sub, subp, rec[l], 0.02, label="scene bf16 L%d" % l, bf16=True)


@pytest.fixture(scope="module")
def vgg_inputs_bf16():
    """Reduced-size replica of the 640x480 VGG-style workload (same recipe and seeds, 64x80,
    4 frames), oracle in bfloat16 mode."""
    cfg = get_config(4, height=64, width=80, n_frames=4)
    params = cfg.weights()
    v = cfg.video()
    frames = [v.frame(t) for t in range(cfg.n_frames)]
    return cfg, params, oracle_layer_inputs(cfg.layers, params, frames, cfg.tau, bf16=True)


@pytest.mark.parametrize("l", [0, 1, 3, 4, 6, 7, 8, 10, 11, 12])
def test_vgg_layer_teacher_forced_bf16(vgg_inputs_bf16, l):
    cfg, params, rec = vgg_inputs_bf16
    sub, subp = _with_pool(cfg.layers, params, l)
    compare_sequence(sub, subp, rec[l], cfg.tau, label="vgg bf16 L%d" % l, bf16=True)


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("hold", [False, True])
def test_random_geometry_bf16(case, hold):
    C, M, kh, kw, s, p, H, W, with_pool = case
    L = type(conv(1, 1, 1))("conv", C, M, kh, kw, s, p, True)
    layers = [L]
    Ho, Wo = (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1
    if with_pool and Ho % 2 == 0 and Wo % 2 == 0:
        layers.append(pool())
    params = make_weights(layers, 7 + C + M)
    v = _video(H, W, C, sigma=0.004, n_objects=2, seed=C * 100 + M)
    frames = [v.frame(t) for t in range(4)]
    compare_sequence(layers, params, frames, 0.015, hold=hold, label="bf16 " + str(case), bf16=True)


@pytest.mark.parametrize("hold", [False, True])
def test_integer_network_every_layer_bit_exact_bf16(hold):
    """Small-integer data: every sum is an exact integer in float32 and in double, and both
    sides round it to bfloat16 the same way, so stored maps and the lists of all layers
    (including those detected inside the producing kernel) must agree bit for bit."""
    layers = [conv(3, 8, 3), pool(), conv(8, 20, 3), conv(20, 12, 1), pool(), conv(12, 5, 3, relu=False)]
    params = _integer_params(layers, 31)
    H, W = 24, 36
    frames = _integer_video(H, W, 3, 7, 77)
    taus = [0.5, None, 1.5, 2.5, None, 3.5]
    net = cb.CBInfer(layers, params, (3, H, W), taus, hold_reference=hold, dtype=cb.BF16)
    orc = oracle.OracleCBNet(layers, params, [0.0 if t is None else t for t in taus], ref_mode=1 if hold else 0,
                             bf16=True)
    sparse_seen = rounded_seen = False
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
            if np.abs(orc.out[l]).max() > 256:
                rounded_seen = True
        np.testing.assert_array_equal(got, want)
    assert sparse_seen, "the deeper layers never saw a sparse change list"
    assert rounded_seen, "no value needed rounding to bfloat16; the test does not exercise it"
    net.destroy()


def test_bf16_threshold_zero_equals_dense_mode_bit_for_bit():
    layers = scene_labeling_net()
    params = make_weights(layers, 5)
    v = _video(48, 64, seed=9)
    a = cb.CBInfer(layers, params, (3, 48, 64), 0.0, dtype=cb.BF16)
    b = cb.CBInfer(layers, params, (3, 48, 64), 0.0, dtype=cb.BF16)
    b.set_mode(True)
    for t in range(4):
        f = to_dev(v.frame(t))
        np.testing.assert_array_equal(a.process_frame(f).cpu().numpy(), b.process_frame(f).cpu().numpy())
    a.destroy()
    b.destroy()


def test_bf16_stored_maps_hold_bfloat16_values():
    cfg = get_config(1)
    net = cb.CBInfer(cfg.layers, cfg.weights(), (3, 64, 64), cfg.tau, dtype=cb.BF16)
    f = cfg.video().frame(0)
    net.process_frame(to_dev(f))
    ref = net.read_map(0, cb.MAP_REFERENCE)[0]
    np.testing.assert_array_equal(ref, oracle.round_bf16(f))
    out = net.read_map(0, cb.MAP_OUTPUT)[0]
    np.testing.assert_array_equal(out, oracle.round_bf16(out))
    net.destroy()


def test_vgg_layer_full_size_sampled_bf16():
    """640x480, 64 -> 64 channels 3x3 (the widest map of the VGG-style workload), bfloat16,
    in the launch configuration the benchmark uses; lists exact, features on sampled positions."""
    cfg = get_config(4)
    L = cfg.layers[1]
    r = np.random.default_rng(cfg.seed(0) + 1)
    w = (r.standard_normal((64, 64, 3, 3)) * np.sqrt(2.0 / (64 * 9))).astype(np.float32)
    b = (r.standard_normal(64) * 0.1).astype(np.float32)
    v = SyntheticVideo(cfg.height, cfg.width, 64, seeds=(cfg.seed(1), cfg.seed(2), cfg.seed(3)), sigma=cfg.sigma,
                       n_objects=5)
    frames = [v.frame(t) for t in range(3)]
    compare_sampled(L, (w, b), frames, cfg.tau, n_samples=400, label="vgg L1 640x480 bf16", bf16=True)


@pytest.mark.parametrize("shape", [
    # C, M, H, W -- the first and the last layer shape of the VGG-style workload
    (3, 64, 480, 640),
    (512, 512, 60, 80),
])
def test_vgg_layer_shapes_full_size_sampled(shape):
    """bfloat16 storage at the workload's full size: exact lists on the whole maps, feature values on
    sampled positions the oracle computes one by one (K = 27 and K = 4608)."""
    from gpu_util import compare_sampled
    from workloads import conv, make_weights
    C, M, H, W = shape
    L = conv(C, M, 3)
    params = make_weights([L], 4000 + C)[0]
    r = np.random.default_rng(C)
    x = r.random((C, H, W), dtype=np.float32)
    seq = [x]
    for t in range(1, 3):
        y = seq[-1].copy()
        for _ in range(6):
            h, w = int(r.integers(3, 12)), int(r.integers(3, 16))
            y0, x0 = int(r.integers(0, H - h)), int(r.integers(0, W - w))
            y[:, y0:y0 + h, x0:x0 + w] = r.random((C, h, w), dtype=np.float32)
        seq.append(y)
    compare_sampled(L, params, seq, 0.05, bf16=True, n_samples=300, label="vgg layer %s" % (shape,))
