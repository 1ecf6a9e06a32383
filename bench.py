#!/usr/bin/env python3
"""Benchmark of the change-based convolution path on one MI355X.

A step is one video frame through the whole hot path (change detection, index extraction,
dilation, gathered matrix multiplication with output update, change propagation through
pooling) of the 320x240 scene-labeling workload.  Frames are synthetic, seeded and already
resident in HBM when the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg1|cfg3|cfg4|cfg5|hbm] [--rate R]
                    [--dtype f32|bf16]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

MI355X_HBM_GBS = 8000.0
MI355X_FP32_MFMA_TFLOPS = 157.3
MI355X_BF16_MFMA_TFLOPS = 2500.0
# HBM bytes per launch of the dominant kernel (gathered GEMM of the 64->256 7x7 layer) on the
# benchmark workload, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by a plain
# copy of known size); the commands and figures are in profiles/cfg2_hbm_traffic.md.
CFG2_DOMINANT_GEMM_HBM_BYTES = 62.6e6


def frame_order(n_frames: int, count: int, start: int = 0):
    """Ping-pong through the sequence so that any number of steps sees ordinary motion."""
    period = 2 * (n_frames - 1)
    for i in range(start, start + count):
        u = i % period
        yield u if u < n_frames else period - u


def build_workload(args):
    from workloads import get_config
    if args.workload == "cfg1":
        cfg = get_config(1)
    elif args.workload == "cfg2":
        cfg = get_config(2)
    elif args.workload == "cfg3":
        cfg = get_config(3, change_rate=args.rate, sigma=args.sigma, n_frames=args.frames or 24)
    elif args.workload == "cfg4":
        cfg = get_config(4, n_frames=args.frames or 24)
    elif args.workload == "cfg5":
        cfg = get_config(5, n_frames=args.frames or 12)
    elif args.workload == "hbm":
        # One 1x1 layer on a 3x4096x4096 frame with a handful of changing pixels: everything but
        # change detection is negligible, and a frame's traffic (~0.7 GB) exceeds the last-level
        # cache, so the detection kernel's rate is an HBM rate.
        from workloads import Config, conv
        cfg = Config("hbm-detect-4096x4096x3", 0, [conv(3, 4, 1, relu=False)], 4096, 4096, 3,
                     args.frames or 3, 0.02, 0.0, video_kwargs={"n_objects": 2})
    else:
        raise SystemExit("unknown workload " + args.workload)
    if args.frames:
        cfg.n_frames = args.frames
    if args.dtype:
        cfg.dtype = args.dtype
    return cfg


def time_steps(net, frames_dev, out, order):
    import torch
    ptrs = [frames_dev[t].data_ptr() for t in order]
    optr = out.data_ptr()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for p in ptrs:
        net.process_frame_ptr(p, optr)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def cpu_baseline(cfg, budget_s: float):
    """The oracle, as it stands, on the host cores.  `value`: its change-based evaluation --
    frame 0 (dense) is processed untimed, then frames 1.. are timed until two thirds of the budget
    are used.  `dense_value`: its stateless per-frame evaluation of the same frames in the rest."""
    import oracle
    params = cfg.weights()
    video = cfg.video()
    net = oracle.OracleCBNet(cfg.layers, params, cfg.tau, bf16=cfg.dtype == "bf16")
    net.process_frame(video.frame(0))
    n, spent = 0, 0.0
    while (spent < budget_s * 2 / 3 and n < cfg.n_frames - 1) or n == 0:
        f = video.frame(n + 1)
        t0 = time.perf_counter()
        net.process_frame(f)
        spent += time.perf_counter() - t0
        n += 1
    nd, spent_d = 0, 0.0
    while (spent_d < budget_s / 3 and nd < cfg.n_frames - 1) or nd == 0:
        f = video.frame(nd + 1)
        t0 = time.perf_counter()
        oracle.dense_forward(cfg.layers, params, f, bf16=cfg.dtype == "bf16")
        spent_d += time.perf_counter() - t0
        nd += 1
    return {"value": n / spent, "unit": "frames/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": "%s frames 1..%d of the same video, change-based oracle (C, double accumulation, "
                      "OpenMP over output positions), frame 0 untimed; dense_value: frames 1..%d through "
                      "the oracle's per-frame dense evaluation" % (cfg.name, n, nd),
            "dense_value": nd / spent_d}


def parse_args(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--rate", type=float, default=0.02, help="cfg3: nominal changed-pixel share")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default=None,
                    help="storage type of maps and weights (default: the workload's)")
    ap.add_argument("--sigma", type=float, default=None, help="override sensor noise")
    ap.add_argument("--hold", action="store_true",
                    help="refresh the stored previous input only where a change was flagged")
    ap.add_argument("--propagate", action="store_true",
                    help="no change detection behind the first layer (worst-case propagation)")
    ap.add_argument("--frames", type=int, default=0, help="frames generated (default: the workload's)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the cpu_baseline leg (0: skip)")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel timing pass")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run three 256 MiB device copies (reference for profiler byte counters)")
    return ap.parse_args(argv)


def run(args) -> dict:
    """One benchmark run; returns the result record that main() prints as a JSON line."""
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one process, one MI355X); --gpus %d is not "
              "supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1704_04313_amd as cb
    from workloads import dense_flops

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    if args.calibrate_copy:
        # a plain device copy of known size (256 MiB read + 256 MiB written) so that HBM byte
        # counters of a profiler run over this process can be scaled
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = build_workload(args)
    params = cfg.weights()
    videos = [cfg.video(s) for s in range(cfg.n_streams)]
    if cfg.n_streams == 1:
        frames = np.stack([videos[0].frame(t) for t in range(cfg.n_frames)])
    else:   # [T][S][C][H][W]: one frame of every stream per step
        frames = np.stack([np.stack([v.frame(t) for v in videos]) for t in range(cfg.n_frames)])
    frames_dev = torch.from_numpy(frames).cuda()
    in_shape = (cfg.channels, cfg.height, cfg.width)
    bf16 = cfg.dtype == "bf16"
    esz = 2.0 if bf16 else 4.0         # bytes per stored map element
    mfma_peak = MI355X_BF16_MFMA_TFLOPS if bf16 else MI355X_FP32_MFMA_TFLOPS
    conv_ids = [l for l, L in enumerate(cfg.layers) if L.kind == "conv"]
    net = cb.CBInfer(cfg.layers, params, in_shape, cfg.tau, n_streams=cfg.n_streams,
                     dtype=cb.BF16 if bf16 else cb.F32, hold_reference=args.hold,
                     propagate_layers=conv_ids[1:] if args.propagate else ())
    out = torch.empty(net.out_shape, dtype=torch.float32, device="cuda")

    W, K = args.warmup, args.steps
    # ---- change-based: warm-up (includes the dense first frame), then exactly K timed steps
    for t in frame_order(cfg.n_frames, W):
        net.process_frame(frames_dev[t], out)
    sec_cb = time_steps(net, frames_dev, out, list(frame_order(cfg.n_frames, K, W)))

    # ---- dense HIP baseline: same kernels, identity lists, no change detection
    net.set_mode(True)
    for t in frame_order(cfg.n_frames, W):
        net.process_frame(frames_dev[t], out)
    sec_dense = time_steps(net, frames_dev, out, list(frame_order(cfg.n_frames, K, W)))
    net.set_mode(False)

    result = {
        "metric": "frames/s and speed-up vs dense HIP conv at 1/5/20% change rate; HBM GB/s",
        "value": cfg.n_streams * K / sec_cb, "unit": "frames/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * sec_cb / K, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "frame": "%dx%dx%d" % (cfg.width, cfg.height, cfg.channels),
                   "tau": cfg.tau, "sigma": cfg.sigma, "n_frames": cfg.n_frames, "n_streams": cfg.n_streams,
                   "reference_update": "where flagged" if args.hold else "previous frame",
                   "detection": "first layer only, changes propagated" if args.propagate else "every layer"},
        "dense_hip_frames_per_s": cfg.n_streams * K / sec_dense,
        "speedup_vs_dense_hip": sec_dense / sec_cb,
        "paper_context": "8.6x (Tegra X1) / 7.6x (GTX 1080) over cuDNN, 327.6 GOp/s/W; other hardware, other data",
    }

    # ---- per-kernel timing pass (HIP events around every launch, on the library's stream)
    if not args.no_profile:
        n_ops = len(cfg.layers)
        net.reset()
        for t in frame_order(cfg.n_frames, W):
            net.process_frame(frames_dev[t], out)
        net.set_profiling(True)
        P = min(K, 100)
        sums = {l: np.zeros(2) for l in range(n_ops)}
        for t in frame_order(cfg.n_frames, P, W):
            net.process_frame(frames_dev[t], out)
            for l in range(n_ops):
                sums[l] += np.maximum(np.array(net.layer_counts(l), dtype=np.float64), 0)
        prof = {}
        for l in range(n_ops):
            for s, name in enumerate(cb.STEP_NAMES):
                ms, n = net.read_profile(l, s)
                if n:
                    prof[(l, name)] = (ms / n, n)
        net.set_profiling(False)
        shapes = [in_shape] + [net.layer_shape(l) for l in range(n_ops)]
        rates, kernels = {}, {}
        for l in range(n_ops):
            L = cfg.layers[l]
            c_in, h_in, w_in = shapes[l]
            c_out, h_out, w_out = shapes[l + 1]
            n_c, n_u = sums[l] / P / cfg.n_streams
            if L.kind == "conv":
                rates["L%d" % l] = {"changed_in": n_c / (h_in * w_in), "updated_out": n_u / (h_out * w_out)}
            else:
                rates["L%d" % l] = {"updated_pooled": n_u / (h_out * w_out)}
            for (ll, name), (ms, n) in prof.items():
                if ll != l:
                    continue
                e = {"us": 1e3 * ms}
                if name == "detect":
                    # frame read (float32) + stored input read and written
                    by = cfg.n_streams * ((4.0 + 2.0 * esz) * c_in * h_in * w_in + h_in * w_in / 8.0)
                    e.update(bytes=by, GBps=by / (ms * 1e-3) / 1e9, frac_hbm=by / (ms * 1e-3) / 1e9 / MI355X_HBM_GBS)
                elif name == "gemm":
                    fl = 2.0 * L.cout * L.cin * L.kh * L.kw * n_u * cfg.n_streams
                    e.update(flops=fl, TFLOPs=fl / (ms * 1e-3) / 1e12,
                             frac_mfma=fl / (ms * 1e-3) / 1e12 / mfma_peak)
                elif name == "compact":
                    by = (h_in * w_in + h_out * w_out) / 8.0 + 4.0 * (n_c + n_u)
                    e.update(bytes=by, GBps=by / (ms * 1e-3) / 1e9)
                elif name == "pool":
                    by = 4.0 * n_u + 5.0 * esz * c_out * n_u
                    e.update(bytes=by, GBps=by / (ms * 1e-3) / 1e9)
                kernels["L%d.%s" % (l, name)] = e
        dom = max(kernels, key=lambda k: kernels[k]["us"])
        d = kernels[dom]
        if "TFLOPs" in d:
            roof = {"bound": "mfma", "achieved": d["TFLOPs"], "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": d["frac_mfma"], "traffic": None}
        else:
            roof = {"bound": "hbm", "achieved": d.get("GBps"), "peak": MI355X_HBM_GBS, "unit": "GB/s",
                    "frac": (d.get("GBps") or 0.0) / MI355X_HBM_GBS, "traffic": None}
        if cfg.name.startswith("cfg2") and dom == "L4.gemm" and not bf16:
            roof["traffic"] = CFG2_DOMINANT_GEMM_HBM_BYTES
        roof["kernel"] = dom
        roof["avg_us"] = d["us"]
        roof["sum_kernel_us_per_frame"] = sum(k["us"] for k in kernels.values())
        result["roofline"] = roof
        result["kernels"] = kernels
        result["change_rates"] = rates
        result["dense_gflop_per_frame"] = sum(dense_flops(cfg.layers, *in_shape)) / 1e9    # per stream
    else:
        result["roofline"] = None

    net.destroy()
    result["cpu_baseline"] = cpu_baseline(cfg, args.cpu_seconds) if args.cpu_seconds > 0 else None
    return result


def main():
    print(json.dumps(run(parse_args())))


if __name__ == "__main__":
    main()
