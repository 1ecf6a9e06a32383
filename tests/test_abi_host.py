"""Host-side checks that need no GPU: the C-ABI library loads, exports every function the
header declares, validates network descriptions, and refuses to run without a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_1704_04313_amd as cb
from paper_1704_04313_amd import binding
from workloads import conv, pool, make_weights, scene_labeling_net

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "cbinfer.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(cbinfer_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_function():
    lib = cb.load_library()
    names = _declared_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_workspace_bytes_and_layout_constants():
    layers = scene_labeling_net()
    n = cb.cbinfer_workspace_bytes(layers, make_weights(layers, 0), (3, 240, 320))
    assert 30e6 < n < 120e6            # maps, lists and 32 MiB of GEMM scratch
    n64 = cb.cbinfer_workspace_bytes(layers, make_weights(layers, 0), (3, 240, 320), n_streams=64)
    assert n64 > 20 * n


def _net_for(layers, params, shape, **kw):
    keep = []
    net = binding._describe(layers, params, shape, kw.get("n_streams", 1), kw.get("flags", 0),
                            kw.get("tau"), (), keep)
    return net, keep


@pytest.mark.parametrize("case,msg", [
    ("cin", "does not match"),
    ("pad", "pad"),
    ("odd_pool", "multiple of the pooling window"),
    ("streams", "n_streams"),
    ("pool_first", "pooling must directly follow"),
    ("dtype", "dtype must be"),
    ("flags", "flag"),
    ("propagate_first", "no op before it"),
    ("propagate_dense", "exclude each other"),
    ("shape", "frame shape"),
])
def test_invalid_descriptions_are_rejected(case, msg):
    lib = cb.load_library()
    layers = [conv(3, 4, 3), pool(), conv(4, 2, 1)]
    shape, kw = (3, 8, 8), {}
    if case == "cin":
        layers = [conv(3, 4, 3), conv(5, 2, 1)]
    elif case == "odd_pool":
        shape = (3, 9, 8)
    elif case == "pool_first":
        layers = [pool(), conv(3, 2, 1)]
    elif case == "streams":
        kw["n_streams"] = 0
    elif case == "flags":
        kw["flags"] = 12
    elif case == "shape":
        shape = (3, 0, 8)
    params = make_weights(layers, 0)
    net, keep = _net_for(layers, params, shape, **kw)
    if case == "pad":
        net.layers[0].pad = 3
    if case == "propagate_first":
        net.layers[0].propagate = 1
    if case == "propagate_dense":
        net.layers[2].propagate = 1
        net.layers[2].dense = 1
    if case == "dtype":
        net.dtype = 7
    assert lib.cbinfer_workspace_bytes(C.byref(net)) == 0
    assert msg in lib.cbinfer_last_error().decode()


def test_null_arguments():
    lib = cb.load_library()
    assert lib.cbinfer_workspace_bytes(None) == 0
    assert lib.cbinfer_process_frame(None, None, None) == -1
    assert lib.cbinfer_reset(None) == -1
    lib.cbinfer_destroy(None)
    assert lib.cbinfer_last_error() is not None


def test_create_fails_loudly_without_a_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    layers = [conv(3, 4, 3)]
    with pytest.raises(cb.CBInferError):
        cb.CBInfer(layers, make_weights(layers, 0), (3, 8, 8), 0.1)
    # and straight through the C ABI
    lib = cb.load_library()
    net, keep = _net_for(layers, make_weights(layers, 0), (3, 8, 8))
    assert not lib.cbinfer_create(C.byref(net), C.c_float(0.1))
    assert b"device" in lib.cbinfer_last_error().lower()


def test_negative_global_threshold_needs_per_layer_values():
    lib = cb.load_library()
    layers = [conv(3, 4, 3)]
    net, keep = _net_for(layers, make_weights(layers, 0), (3, 8, 8))
    assert not lib.cbinfer_create(C.byref(net), C.c_float(float("nan")))
    assert b"threshold" in lib.cbinfer_last_error()


def test_oversize_maps_are_refused_not_truncated():
    """Pixel indices and element offsets are 32-bit inside the kernels: a map beyond 2^31 - 1
    elements must be refused when the network is described, whatever the device could hold."""
    lib = cb.load_library()
    layers = [conv(3, 8, 3)]
    net, keep = _net_for(layers, make_weights(layers, 0), (3, 40000, 40000))
    assert lib.cbinfer_workspace_bytes(C.byref(net)) == 0
    assert "2^31-1" in lib.cbinfer_last_error().decode()
    # many streams of an ordinary frame overflow the same limit
    net, keep = _net_for(layers, make_weights(layers, 0), (3, 1080, 1920), n_streams=400)
    assert lib.cbinfer_workspace_bytes(C.byref(net)) == 0


def test_workspace_grows_with_streams_and_shrinks_with_bfloat16():
    layers = [conv(3, 16, 7), pool(), conv(16, 32, 3)]
    params = make_weights(layers, 1)
    one = cb.cbinfer_workspace_bytes(layers, params, (3, 240, 320))
    four = cb.cbinfer_workspace_bytes(layers, params, (3, 240, 320), n_streams=4)
    half = cb.cbinfer_workspace_bytes(layers, params, (3, 240, 320), dtype=cb.BF16)
    assert four > 2 * one > 0
    assert half < one


def test_large_three_channel_frames_are_stored_without_a_padding_channel():
    """From 2^18 pixels on a float32 frame with 3 channels keeps 3 values per pixel in the stored
    previous input (the detection pass then moves no padding); smaller frames, four channels and
    bfloat16 keep whole 16-byte units.  Seen from the host through the workspace size."""
    def ws(c, h, w, **kw):
        layers = [conv(c, 8, 3)]
        return cb.cbinfer_workspace_bytes(layers, make_weights(layers, 2), (c, h, w), **kw)

    big = 512 * 512                                   # = 2^18 pixels
    saved = ws(4, 512, 512) - ws(3, 512, 512)
    assert big * 4 <= saved < big * 4 + 4096          # one float per pixel less, nothing else differs
    assert ws(4, 256, 256) == ws(3, 256, 256)         # small frames: padded either way
    assert ws(4, 512, 512, dtype=cb.BF16) == ws(3, 512, 512, dtype=cb.BF16)
    held = ws(4, 512, 512, flags=cb.FLAG_HOLD_REFERENCE) - ws(3, 512, 512, flags=cb.FLAG_HOLD_REFERENCE)
    assert 2 * big * 4 <= held < 2 * big * 4 + 8192   # hold mode keeps two such maps


def test_static_workspace_size_limit_is_checked_before_any_device_call():
    """cbinfer_create_static keeps a network's state in a device array of fixed size inside the
    library: a network that needs more is refused with a message that names both sizes, and the
    320x240 scene-labeling network (the benchmark workload) fits."""
    lib = cb.load_library()
    cap = lib.cbinfer_static_workspace_bytes()
    assert cap == 64 << 20
    layers = scene_labeling_net()
    params = make_weights(layers, 0)
    assert cb.cbinfer_workspace_bytes(layers, params, (3, 240, 320)) <= cap
    net, keep = _net_for(layers, params, (3, 720, 1280))
    need = lib.cbinfer_workspace_bytes(C.byref(net))
    assert need > cap
    assert not lib.cbinfer_create_static(C.byref(net), C.c_float(0.02))
    msg = lib.cbinfer_last_error().decode()
    assert str(need) in msg and str(cap) in msg
    # an invalid description is rejected the same way cbinfer_create rejects it
    net, keep = _net_for([conv(3, 4, 3), conv(5, 2, 1)], make_weights([conv(3, 4, 3), conv(5, 2, 1)], 0), (3, 8, 8))
    assert not lib.cbinfer_create_static(C.byref(net), C.c_float(0.02))
    assert "does not match" in lib.cbinfer_last_error().decode()
