#!/usr/bin/env python3
"""Speed-up against change rate: the 1280x720 scene-labeling workload with the number of moving
objects chosen per nominal share of changed pixels (0.5, 2, 10, 30 %, and 100 % = a new background
every frame), once without sensor noise and once with sigma = 0.005.  Prints a markdown table; each
row is one bench.py run (same timing rules: frames resident in HBM, change-based frames/s against
the dense HIP baseline of the same library).

    python bench_sweep.py [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import sys

import bench


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--rates", default="0.005,0.02,0.1,0.3,1.0")
    ap.add_argument("--sigmas", default="0,0.005")
    ap.add_argument("--json", default="", help="also write every run's record to this file")
    a = ap.parse_args()
    rows, records = [], []
    for sigma in [float(v) for v in a.sigmas.split(",")]:
        for rate in [float(v) for v in a.rates.split(",")]:
            args = bench.parse_args(["--workload", "cfg3", "--rate", str(rate), "--sigma", str(sigma), "--steps",
                                     str(a.steps), "--warmup", str(a.warmup), "--cpu-seconds", "0"])
            r = bench.run(args)
            records.append(r)
            cr = r["change_rates"]
            upd = [cr[k].get("updated_out", cr[k].get("updated_pooled")) for k in sorted(cr)]
            g = r["kernels"].get("L4.gemm", {})
            rows.append("| %g | %g | %.2f %% | %s | %.0f | %.0f | %.2fx | %.1f |" % (
                rate * 100, sigma, 100 * cr["L0"]["changed_in"],
                " / ".join("%.1f" % (100 * u) for i, u in enumerate(upd) if "updated_out" in cr[sorted(cr)[i]]),
                r["value"], r["dense_hip_frames_per_s"], r["speedup_vs_dense_hip"], g.get("TFLOPs", 0.0)))
            print(rows[-1], file=sys.stderr, flush=True)
    print("| nominal changed % | sigma | measured changed input pixels | outputs recomputed per conv layer % "
          "| change-based frames/s | dense HIP frames/s | speed-up | 64->256 7x7 GEMM TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|")
    print("\n".join(rows))
    if a.json:
        with open(a.json, "w") as f:
            json.dump(records, f)


if __name__ == "__main__":
    main()
