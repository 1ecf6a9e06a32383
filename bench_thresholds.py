#!/usr/bin/env python3
"""Threshold study on synthetic video (the experiment of Section 4.3 in kind): the per-layer
change-detection thresholds are scaled jointly by a factor 0 ... 2 and, per factor, the share of
changed inputs and recomputed outputs of every convolution layer, the frame rate and the deviation
of the network output from per-frame dense inference are reported.

Base thresholds: the workload's threshold for the first layer; for every deeper layer the same
value scaled by the ratio of that layer's mean absolute input to the frame's, measured once on
frame 0 (thresholds that grow with the depth of the layer, as the values selected in Section 4.3
do).  Optionally every layer behind the first takes its changes from the layer before it without
a detection of its own (worst-case propagation, Section 4.7), and the reference-update variant
can be selected.  From the command line the dense result comes from the dense mode of the same
library; study() takes the per-frame dense results from its caller, and
tests/test_gpu_threshold_study.py passes it the CPU oracle's on a prefix of the video.  Prints a
markdown table.

    python bench_thresholds.py [--workload cfg2] [--frames 40] [--factors 0,0.25,...] [--propagate] [--hold]
"""
from __future__ import annotations

import argparse
import sys
import time

import numpy as np


def layer_scales(cfg, params, frames, dtype):
    """Dense-mode outputs of every frame and the mean absolute input of every convolution layer on frame 0."""
    import paper_1704_04313_amd as cb
    in_shape = (cfg.channels, cfg.height, cfg.width)
    conv_ids = [l for l, L in enumerate(cfg.layers) if L.kind == "conv"]
    dense = cb.CBInfer(cfg.layers, params, in_shape, 0.0, dtype=dtype)
    dense.set_mode(True)
    ref_out = [dense.process_frame(frames[t]).clone() for t in range(frames.shape[0])]
    dense.process_frame(frames[0])
    scale = {conv_ids[0]: float(frames[0].abs().mean())}
    for l in conv_ids[1:]:
        scale[l] = float(np.abs(dense.read_map(l - 1, cb.MAP_OUTPUT)).mean())
    dense.destroy()
    return ref_out, scale


def study(cfg, params, frames, ref_out, base, factors, *, dtype, propagate=False, hold=False, timing=True):
    """One row per factor: the thresholds base[l] * factor, the change-based network run over
    `frames` (device tensor [T][C][H][W]) and compared frame by frame (from frame 1 on) with
    `ref_out` -- the per-frame dense results, one device tensor per frame, from whatever
    evaluates them (the library's dense mode, or the caller's own reference)."""
    import torch
    import bench
    import paper_1704_04313_amd as cb
    in_shape = (cfg.channels, cfg.height, cfg.width)
    conv_ids = [l for l, L in enumerate(cfg.layers) if L.kind == "conv"]
    T = frames.shape[0]
    rows = []
    for fac in factors:
        taus = [fac * base[l] if l in base else None for l in range(len(cfg.layers))]
        net = cb.CBInfer(cfg.layers, params, in_shape, taus, dtype=dtype, hold_reference=hold,
                         propagate_layers=conv_ids[1:] if propagate else ())
        out = torch.empty(net.out_shape, dtype=torch.float32, device="cuda")
        n_c = {l: 0.0 for l in conv_ids}
        n_u = {l: 0.0 for l in conv_ids}
        max_err, se, sr, agree, total = 0.0, 0.0, 0.0, 0.0, 0.0
        for t in range(T):
            net.process_frame(frames[t], out)
            if t == 0:
                continue
            d = out - ref_out[t]
            max_err = max(max_err, float(d.abs().max()))
            se += float((d.double() ** 2).sum())
            sr += float((ref_out[t].double() ** 2).sum())
            agree += float((out.argmax(dim=1) == ref_out[t].argmax(dim=1)).sum())
            total += out.shape[0] * out.shape[2] * out.shape[3]
            for l in conv_ids:
                c, u = net.layer_counts(l)
                n_c[l] += c
                n_u[l] += u
        shapes = [in_shape] + [net.layer_shape(l) for l in range(len(cfg.layers))]
        row = {"factor": fac,
               "changed_in": [n_c[l] / (T - 1) / (shapes[l][1] * shapes[l][2]) for l in conv_ids],
               "updated_out": [n_u[l] / (T - 1) / (shapes[l + 1][1] * shapes[l + 1][2]) for l in conv_ids],
               "max_abs_error": max_err, "rms_rel_error": (se / sr) ** 0.5 if sr else 0.0,
               "label_agreement": agree / total, "frames_per_s": None}
        if timing:  # the same frames again (ping-pong order), nothing read back
            order = list(bench.frame_order(T, 3 * T, 1))
            for t in order[:10]:
                net.process_frame(frames[t], out)
            row["frames_per_s"] = len(order) / bench.time_steps(net, frames, out, order)
        net.destroy()
        rows.append(row)
    return rows


def format_rows(rows):
    lines = ["| factor | changed inputs per conv layer % | outputs recomputed per conv layer % | frames/s | "
             "max abs error | rms error / rms output | label agreement % |", "|---|---|---|---|---|---|---|"]
    for r in rows:
        lines.append("| %.2f | %s | %s | %s | %.3g | %.3g | %.2f |" % (
            r["factor"], " / ".join("%.1f" % (100 * v) for v in r["changed_in"]),
            " / ".join("%.1f" % (100 * v) for v in r["updated_out"]),
            "-" if r["frames_per_s"] is None else "%.0f" % r["frames_per_s"], r["max_abs_error"],
            r["rms_rel_error"], 100.0 * r["label_agreement"]))
    return lines


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--frames", type=int, default=40)
    ap.add_argument("--factors", default="0,0.25,0.5,0.75,1,1.25,1.5,1.75,2")
    ap.add_argument("--flat", action="store_true", help="same base threshold in every layer")
    ap.add_argument("--propagate", action="store_true", help="no detection behind the first layer")
    ap.add_argument("--hold", action="store_true", help="refresh the stored input only where flagged")
    ap.add_argument("--sigma", type=float, default=None)
    a = ap.parse_args()

    import torch
    import bench
    import paper_1704_04313_amd as cb

    if not torch.cuda.is_available():
        print("bench_thresholds.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    cfg = bench.build_workload(bench.parse_args(["--workload", a.workload, "--frames", str(a.frames)] +
                                                (["--sigma", str(a.sigma)] if a.sigma is not None else [])))
    if cfg.n_streams != 1:
        raise SystemExit("single-stream workloads only")
    params = cfg.weights()
    video = cfg.video()
    frames = torch.from_numpy(np.stack([video.frame(t) for t in range(cfg.n_frames)])).cuda()
    conv_ids = [l for l, L in enumerate(cfg.layers) if L.kind == "conv"]
    dtype = cb.BF16 if cfg.dtype == "bf16" else cb.F32
    ref_out, scale = layer_scales(cfg, params, frames, dtype)
    base = {l: cfg.tau * (1.0 if a.flat else scale[l] / scale[conv_ids[0]]) for l in conv_ids}

    print("workload %s, %d frames, sigma %g, base thresholds %s%s%s" % (
        cfg.name, cfg.n_frames, cfg.sigma, ", ".join("L%d %.4g" % (l, base[l]) for l in conv_ids),
        ", worst-case propagation behind the first layer" if a.propagate else "",
        ", reference refreshed only where flagged" if a.hold else ""))
    print()
    rows = study(cfg, params, frames, ref_out, base, [float(v) for v in a.factors.split(",")], dtype=dtype,
                 propagate=a.propagate, hold=a.hold)
    print("\n".join(format_rows(rows)), flush=True)


if __name__ == "__main__":
    main()
