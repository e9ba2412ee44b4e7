"""Writes the head-bias calibration files of the full-size workloads (TEST INFRASTRUCTURE; calls only the oracle and
the input generators).  Usage: python -m oracle.calibrate_configs config2 [config3 ...] [--n-cal N]

Random-weight experts on noise images route every request the same way unless the routing experts' head biases are
offset.  The offsets are computed here from oracle logits on calibration images whose request ids never coincide
with workload requests, and stored next to the generators; both the HIP path and the oracle then read them as inputs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import guard as G  # noqa: E402
import coe_workloads as W  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("configs", nargs="+")
    ap.add_argument("--n-cal", type=int, default=256)
    ap.add_argument("--out-dir", default=W._CALIB_DIR, help="where the .json files go (default: next to the generators)")
    args = ap.parse_args()
    os.makedirs(args.out_dir, exist_ok=True)
    for name in args.configs:
        t0 = time.time()
        if name == "config2":
            wl, targets = W.config2(calibrated=False), None
        elif name == "config3":
            wl = W.config3(calibrated=False)
            targets = {0: W.zipf_probs(63, 1.1)}
        elif name == "config4":
            wl, targets = W.config4(calibrated=False), None
        elif name == "config5":
            wl, targets = W.config5(calibrated=False), None
        elif name == "config6":
            wl, targets = W.config6(calibrated=False), None
        else:
            raise SystemExit(f"unknown config {name}")
        hb = G.calibrate_workload(wl, n_cal=args.n_cal, targets=targets,
                                  progress=lambda e: print(f"  {name}: expert {e} calibrated ({time.time() - t0:.0f}s)", flush=True))
        out = {"workload": wl.name, "seed": wl.seed, "n_cal": args.n_cal, "input_kind": wl.input_kind,
               "head_bias": {str(e): [float(v) for v in b] for e, b in hb.items()}}
        path = os.path.join(args.out_dir, wl.name + ".json")
        with open(path, "w") as f:
            json.dump(out, f, indent=0)
        print(f"{name}: {len(hb)} routing experts calibrated on {args.n_cal} images in {time.time() - t0:.1f}s -> {path}", flush=True)


if __name__ == "__main__":
    main()
