"""Writes wind_inputs/calibration.json: per workload, the blank-logit bias that makes the stated
fraction of the sequential decoder's joiner evaluations return blank.

Run as `python -m oracle.calibrate [config ...]`.  Calls only the CPU oracle.  The workloads'
"~85 % of frames predict blank" is read as: blank evaluations / all evaluations of Algorithm 1.
The bias is found by bisection on a sub-sample (16 utterances x 600 frames, or the whole workload
if it is smaller: frames that carry the full S labels weigh heavily in the rate, and a smaller sample
holds too few of them to stand for the workload); the achieved rate and the histogram of labels per emitting frame are stored
next to it for the record.  `pred_gain` (a gain on the prediction projection, so that a label
changes the logits enough for the frame that emitted it to turn blank again) is fixed by hand.
"""
from __future__ import annotations

import json
import os
import sys

import numpy as np

import oracle
import wind_inputs as wi

PRED_GAIN = {"tiny": 4.0, "greedy_b1": 4.0, "batch32": 4.0, "largevocab_b128": 4.0, "lowblank_b256": 4.0}
OUT = os.path.join(os.path.dirname(os.path.abspath(wi.__file__)), "calibration.json")


def measure(cfg, enc, lens, bias, gain):
    w = wi.make_weights(cfg, blank_bias=bias, pred_gain=gain)
    o = oracle.Oracle.from_config(cfg, w)
    _, frs, logs = o.greedy_batch(enc, lens, cfg.S, want_log=True)
    ev = sum(len(l) for l in logs)
    bl = sum(int((l["label"] == cfg.V).sum()) for l in logs)
    per = [np.bincount(f)[np.bincount(f) > 0] for f in frs if len(f)]
    per = np.concatenate(per) if per else np.zeros(0, int)
    hist = np.bincount(per, minlength=cfg.S + 1)[1:]
    return bl / max(ev, 1), hist.tolist()


def calibrate(name: str) -> dict:
    cfg = wi.CONFIGS[name]
    sub = cfg if cfg.B * cfg.len_hi <= 9600 else wi.scaled(cfg, 16, 600, 600)
    enc, lens = wi.make_batch(sub)
    gain = PRED_GAIN[name]
    lo, hi = -4.0, 16.0
    for _ in range(16):
        mid = 0.5 * (lo + hi)
        rate, hist = measure(cfg, enc, lens, mid, gain)
        print(f"  {name}: bias {mid:.4f} -> blank rate {rate:.4f}", flush=True)
        if abs(rate - cfg.blank_rate) < 0.003:
            lo = hi = mid
            break
        if rate < cfg.blank_rate:
            lo = mid
        else:
            hi = mid
    bias = round(0.5 * (lo + hi), 4)
    rate, hist = measure(cfg, enc, lens, bias, gain)
    return {"blank_bias": bias, "pred_gain": gain, "subsample": [int(sub.B), int(sub.len_lo)],
            "achieved_blank_rate": round(rate, 4), "labels_per_emitting_frame_hist": hist}


def main(argv):
    names = argv or list(wi.CONFIG_ORDER)
    table = wi.load_calibration()
    for n in names:
        table[n] = calibrate(n)
        print(n, table[n], flush=True)
    with open(OUT, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main(sys.argv[1:])
