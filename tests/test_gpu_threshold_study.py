"""The threshold study (the experiment of Section 4.3 in kind) with the error measured against the
CPU oracle's per-frame dense inference instead of the library's own dense mode: the 320x240
benchmark workload at full size, frames 0..5, thresholds scaled jointly by 0, 0.5, 1, 1.25 and 2.
Checks what the method promises -- factor 0 reproduces dense inference (Section 3.3), the error
grows with the factor and stays small against the output while the recomputed share falls -- and
leaves the table in the file that the environment variable CBINFER_STUDY_TABLE names, if set."""
import os

import numpy as np
import pytest

import oracle
import paper_1704_04313_amd as cb
from workloads import get_config

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_threshold_study_error_against_the_oracles_dense_inference():
    import torch
    import bench_thresholds as bt
    cfg = get_config(2, n_frames=6)
    params = cfg.weights()
    video = cfg.video()
    host = [video.frame(t) for t in range(cfg.n_frames)]
    frames = torch.from_numpy(np.stack(host)).cuda()
    want = [oracle.dense_forward(cfg.layers, params, f)[-1] for f in host]            # O-dense, every frame
    ref_out = [torch.from_numpy(w[None]).cuda() for w in want]
    conv_ids = [l for l, L in enumerate(cfg.layers) if L.kind == "conv"]
    lib_dense, scale = bt.layer_scales(cfg, params, frames, cb.F32)
    # the library's dense mode against the oracle's, the stated float32 tolerance
    for t in range(cfg.n_frames):
        a, b = lib_dense[t].cpu().numpy()[0], want[t]
        assert np.all(np.abs(a - b) <= 1e-5 + 1e-4 * np.abs(b)), "dense mode frame %d" % t
    base = {l: cfg.tau * scale[l] / scale[conv_ids[0]] for l in conv_ids}
    factors = [0.0, 0.5, 1.0, 1.25, 2.0]
    rows = bt.study(cfg, params, frames, ref_out, base, factors, dtype=cb.F32, timing=False)
    r = {row["factor"]: row for row in rows}
    # threshold zero: everything recomputed, dense inference reproduced to rounding
    assert all(u == 1.0 for u in r[0.0]["updated_out"])
    assert r[0.0]["rms_rel_error"] < 1e-6 and r[0.0]["label_agreement"] == 1.0
    # larger thresholds: less is recomputed, the deviation grows, labels hardly move
    assert r[2.0]["updated_out"][0] < r[1.0]["updated_out"][0] < r[0.5]["updated_out"][0] <= 1.0
    assert r[0.5]["rms_rel_error"] <= r[1.0]["rms_rel_error"] <= r[2.0]["rms_rel_error"] < 0.05
    assert r[1.25]["updated_out"][0] < 0.2 and r[1.25]["label_agreement"] > 0.99
    table = os.environ.get("CBINFER_STUDY_TABLE")
    if table:
        with open(table, "w") as f:
            f.write("workload %s, frames 1..%d against the CPU oracle's per-frame dense inference, base thresholds %s\n\n"
                    % (cfg.name, cfg.n_frames - 1, ", ".join("L%d %.4g" % (l, base[l]) for l in conv_ids)))
            f.write("\n".join(bt.format_rows(rows)) + "\n")
