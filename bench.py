#!/usr/bin/env python3
"""Benchmark of the WIND greedy-decoding hot path on one MI355X.

A step is one wind_greedy_decode call over one batch of synthetic encoder outputs that already
sit in HBM: encoder projection, then the loop of window gather, output contraction with row
argmax, first-non-blank decision, pointer update and prediction-network step until every
utterance is done.  The headline workload is benchmark configs[1] (B=1, T=1000, the window
sweep of the paper's Table 1); the roofline object is measured on configs[3] (B=128, V=8192),
the workload on which the joint kernel is MFMA-bound.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FRAME_SECONDS = 0.080          # configs[1]: 80 ms of audio per encoder frame
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def timed_decodes(torch, model, d_enc, d_len, W, S, steps, warmup, out):
    tok, frm, cnt = out
    for _ in range(warmup):
        model.greedy_decode(d_enc, d_len, W, S, tok, frm, cnt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        model.greedy_decode(d_enc, d_len, W, S, tok, frm, cnt)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def run_workload(torch, wi, WindModel, name, windows, steps, warmup, with_sequential):
    cfg = wi.CONFIGS[name]
    w = wi.make_weights(cfg)
    enc, lens = wi.make_batch(cfg)
    frames = int(lens.sum())
    model = WindModel.from_config(cfg, w)
    d_enc = torch.from_numpy(enc).cuda()
    d_len = torch.from_numpy(lens).cuda()
    B, T, _ = enc.shape
    cap = T * cfg.S
    out = (torch.zeros((B, cap), dtype=torch.int32, device="cuda"),
           torch.zeros((B, cap), dtype=torch.int32, device="cuda"),
           torch.zeros((B,), dtype=torch.int32, device="cuda"))
    res = {}
    ws = list(windows or cfg.windows)
    for W in ([None] if with_sequential else []) + ws:
        cold = None
        if not res:
            # the model's first call: workspace allocation, graph capture and instantiation, no launch-ahead
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            model.greedy_decode(d_enc, d_len, W, cfg.S, *out)
            torch.cuda.synchronize()
            cold = (time.perf_counter() - t0) * 1e3
        sec = timed_decodes(torch, model, d_enc, d_len, W, cfg.S, steps, warmup, out)
        st = model.stats()
        res["seq" if W is None else str(W)] = {
            **({"cold_first_call_ms": cold} if cold is not None else {}),
            "frames_per_s": frames / sec, "rtfx": frames * FRAME_SECONDS / sec, "ms_per_step": sec * 1e3,
            "iterations": int(st.iterations), "rows": int(st.rows), "useful_rows": int(st.useful_rows),
            "labels": int(st.labels), "rechecks": int(st.rechecks),
            # pointer advance per window, 0..W (Analysis, Jump Distribution)
            "jump_hist": [int(x) for x in st.jump_hist[:(1 if W is None else W) + 1]]}
    # what the synthetic workload turned out to be (the configurations state targets): blank share of the
    # standard loop's joiner evaluations, and how many labels the emitting frames carry
    import numpy as np

    cnt = out[2].cpu().numpy()
    frm = out[1].cpu().numpy()
    per_frame = np.zeros(cfg.S + 1, np.int64)
    for b in range(B):
        if cnt[b]:
            per_frame += np.bincount(np.bincount(frm[b, : cnt[b]]), minlength=cfg.S + 1)[: cfg.S + 1]
    per_frame[0] = 0
    evals = frames + int(st.labels) - int(st.forced_advances)
    res["workload_stats"] = {
        "blank_share_of_evaluations": round((frames - int(st.forced_advances)) / max(evals, 1), 4),
        "target_blank_share": cfg.blank_rate, "labels": int(st.labels), "forced_advances": int(st.forced_advances),
        "emitting_frames_by_label_count": {str(k): int(v) for k, v in enumerate(per_frame) if k and v}}
    return cfg, model, (d_enc, d_len, out), frames, res, (enc, lens, w)


KERNEL_SOURCES = tuple("paper_2505_13765_amd/csrc/" + f for f in (
    "wind_types.h", "wind_enc_kernels.h", "wind_joint_kernels.h", "wind_mfma_ws.h", "wind_mfma_wide.h", "wind_mfma_dma.h", "wind_util.h"))


def kernel_source_digest():
    """One hash over the kernel sources: a counter summary under profiles/ names the digest it was measured at."""
    import hashlib

    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(cfg, W):
    """HBM bytes per joint launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE runs,
    scaled by a copy kernel of known size), and whether that summary was measured on the kernel sources as
    they are now.  A summary of older kernels is not reported as this build's traffic."""
    path = os.path.join(ROOT, "profiles", f"joint_hbm_traffic_{cfg.name}_w{W}.txt")
    if not os.path.exists(path):
        return None, "no counter summary for this workload"
    traffic, digest = None, None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            traffic = float(line.split(":")[1])
        if line.startswith("kernel_source_digest:"):
            digest = line.split(":")[1].strip()
    if digest != kernel_source_digest():
        return None, f"summary measured at kernel sources {digest}, these are {kernel_source_digest()}: stale, not reported"
    return traffic, f"measured at kernel sources {digest} (current)"


def roofline_leg(torch, cfg, model, dev, W):
    """Times every kernel launch of one decode with events (the library's profile mode) and prices
    the joint kernel against the bf16 MFMA peak: algorithmic flops = 2 * Hj * (V+1) per window row
    the method evaluates (rows past an utterance's end and tile padding do not count)."""
    d_enc, d_len, out = dev
    model.set_option("profile", 1)
    model.greedy_decode(d_enc, d_len, W, cfg.S, *out)     # warm (allocations)
    model.set_option("profile", 1)                        # resets the accumulators
    model.greedy_decode(d_enc, d_len, W, cfg.S, *out)
    st = model.stats()
    kt = model.kernel_times()
    rows_l, us_l = model.joint_launches()
    model.set_option("profile", 0)
    ms, n = kt["joint"]
    # the same figure by row count: launches of the decode binned by the window rows they evaluated
    per_row = 2.0 * cfg.Hj * (cfg.V + 1)
    edges = [0, 128, 256, 384, 512, 768, 1024, 1280, 1536, 1792, 2048, 3072, 4096]
    buckets = []
    for lo, hi in zip(edges[:-1], edges[1:]):
        sel = [(r, u) for r, u in zip(rows_l, us_l) if lo < r <= hi]
        if not sel:
            continue
        r_sum, u_sum = sum(r for r, _ in sel), sum(u for _, u in sel)
        tf = per_row * r_sum / (u_sum * 1e-6) / 1e12
        buckets.append({"rows": f"{lo + 1}-{hi}", "launches": len(sel), "avg_rows": round(r_sum / len(sel), 1),
                        "avg_us": round(u_sum / len(sel), 2), "share_of_time": round(u_sum / max(sum(us_l), 1e-9), 3),
                        "tflops": round(tf, 1), "frac": round(tf / PEAK_BF16_TFLOPS, 3)})
    flops = 2.0 * cfg.Hj * (cfg.V + 1) * st.rows
    achieved = flops / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
    # bytes the joint kernel must move per launch: W_out once, the window rows once, the keys out
    traffic, traffic_note = measured_traffic(cfg, W)
    rows_per_launch = st.rows / max(n, 1)
    # iterations above this many window rows run joint_wide_kernel (256-column tiles of at least 192 rows), the rest joint_ws_kernel
    nt_wide = (cfg.V + 255) // 256
    wide_rows = 128 * max(1, 256 // nt_wide)
    n_wide = sum(1 for r in rows_l if r > wide_rows)
    algorithmic_bytes = cfg.Hj * (cfg.V + 1) * 2 + rows_per_launch * cfg.Hj * 2 + rows_per_launch * ((cfg.V + 63) // 64) * 16
    return {
        "bound": "mfma", "kernel": "joint_ws_kernel + joint_wide_kernel", "workload": f"{cfg.name} W={W}",
        "kernel_split": {"joint_wide_kernel": {"rows_above": wide_rows, "launches": n_wide},
                         "joint_ws_kernel": {"launches": len(rows_l) - n_wide}},
        "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
        "traffic": traffic, "traffic_source": traffic_note,
        "hbm_frac": (traffic / (ms * 1e-3 / max(n, 1)) / 1e9 / PEAK_HBM_GBS) if traffic else None,
        "launches": int(n), "avg_launch_us": ms * 1e3 / max(n, 1),
        "rows_per_launch": rows_per_launch, "flops_per_row": 2.0 * cfg.Hj * (cfg.V + 1),
        "algorithmic_bytes_per_launch": round(algorithmic_bytes),
        "kernel_ms": {k: round(v[0], 3) for k, v in kt.items()},
        "kernel_launches": {k: int(v[1]) for k, v in kt.items()},
        "by_rows": buckets,
    }


def graph_ablation(torch, wi, WindModel, steps, warmup):
    """The structure of the paper's graph ablation (Analysis, Incorporation with CUDA-graphs, Table 5: batch 16,
    the standard loop against window 8, each with and without graph replay) on the batch32 model cut to 16
    utterances.  Three ways to run the same kernels: "eager" = launched one by one with the host waiting for
    every iteration and reading the active count before it launches the next (what a framework loop without
    graphs does, the table's rows without graph); "launches" = one by one, the host polling once per 16
    iterations; "graph" = 16 iterations per graph replay, same polling.  Per cell: wall time of a whole call,
    and the loop alone on the device's clock (the table's decoder-only time; the total here adds only the
    encoder projection and the start-token step, the paper's total adds the whole encoder)."""
    cfg = wi.scaled(wi.CONFIGS["batch32"], 16, wi.CONFIGS["batch32"].len_lo, wi.CONFIGS["batch32"].len_hi)
    w = wi.make_weights(cfg)
    enc, lens = wi.make_batch(cfg)
    model = WindModel.from_config(cfg, w)
    d_enc = torch.from_numpy(enc).cuda()
    d_len = torch.from_numpy(lens).cuda()
    B, T, _ = enc.shape
    cap = T * cfg.S
    out = (torch.zeros((B, cap), dtype=torch.int32, device="cuda"),
           torch.zeros((B, cap), dtype=torch.int32, device="cuda"),
           torch.zeros((B,), dtype=torch.int32, device="cuda"))
    res = {"workload": f"batch32 model, B=16, {int(lens.sum())} frames", "unit": "ms per decode call",
           "paper_table5_decoder_only_s": {"standard": {"eager": 12.45, "graph": 4.23}, "wind_w8": {"eager": 6.45, "graph": 2.10},
                                           "hardware": "2x A6000, Parakeet-RNNT-1.1b, real audio"}}
    for name, W in (("standard", None), ("wind_w8", 8)):
        row = {}
        for mode, opts in (("eager", {"host_sync": 1, "graph": 0}), ("launches", {"host_sync": 0, "graph": 0}),
                           ("graph", {"host_sync": 0, "graph": 1})):
            for k, v in opts.items():
                model.set_option(k, v)
            wall = timed_decodes(torch, model, d_enc, d_len, W, cfg.S, steps, warmup, out) * 1e3
            total, loop = model.call_times()
            row[mode] = {"wall": round(wall, 3), "loop_only": round(loop, 3), "iterations": int(model.stats().iterations)}
        res[name] = row
    res["loop_only_speedup"] = {
        "window_eager": round(res["standard"]["eager"]["loop_only"] / res["wind_w8"]["eager"]["loop_only"], 2),
        "window_graph": round(res["standard"]["graph"]["loop_only"] / res["wind_w8"]["graph"]["loop_only"], 2),
        "graph_standard": round(res["standard"]["eager"]["loop_only"] / res["standard"]["graph"]["loop_only"], 2),
        "graph_wind": round(res["wind_w8"]["eager"]["loop_only"] / res["wind_w8"]["graph"]["loop_only"], 2),
        "both": round(res["standard"]["eager"]["loop_only"] / res["wind_w8"]["graph"]["loop_only"], 2),
        "paper": {"window_eager": 1.93, "window_graph": 2.01, "graph_standard": 2.94, "graph_wind": 3.07, "both": 5.93}}
    model.set_option("host_sync", 0)
    model.set_option("graph", 1)
    model.close()
    return res


def beam_scoring(torch, wi, WindModel, steps):
    """Time of the beam-search scoring step (Eq. 1 and lines 10-13 of Algorithm 3) on the headline
    model: 16 hypotheses on a window of 16 frames, 8 expansions each.  Whole calls, device-resident
    inputs and outputs; the call waits for completion."""
    import numpy as np

    cfg = wi.CONFIGS["greedy_b1"]
    w = wi.make_weights(cfg)
    model = WindModel.from_config(cfg, w)
    rng = np.random.default_rng(5)
    Bh, n, K = 16, 16, 8
    win = torch.from_numpy(wi.round_to_bf16(rng.normal(size=(n, cfg.D)).astype(np.float32))).cuda()
    g = torch.from_numpy(np.tanh(rng.normal(size=(Bh, cfg.Hp))).astype(np.float32)).cuda()
    out = (torch.zeros((Bh, K), dtype=torch.int32, device="cuda"), torch.zeros((Bh, K), dtype=torch.int32, device="cuda"),
           torch.zeros((Bh, K), dtype=torch.float32, device="cuda"))
    for _ in range(3):
        model.beam_window_scores(win, g, K, out)
    torch.cuda.synchronize()
    reps = max(10, steps * 10)
    t0 = time.perf_counter()
    for _ in range(reps):
        model.beam_window_scores(win, g, K, out)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / reps
    model.close()
    return {"workload": f"greedy_b1 model, {Bh} hypotheses x {n} frames, K={K}", "us_per_call": round(sec * 1e6, 2),
            "rows": Bh * n, "logit_bytes": Bh * n * (cfg.V + 1) * 4,
            "joiner_gflops": round(2.0 * Bh * n * cfg.Hj * (cfg.V + 1) / 1e9, 3)}


def beam_search(torch, wi, WindModel):
    """Whole WIND beam search (Algorithm 3) on the first 250 frames of the headline utterance: beam 4,
    window 16 against window 1, in both logit modes (bf16 MFMA pass; fp32 hidden vector).  One call
    each after a warm-up call; device-resident encoder outputs."""
    cfg = wi.CONFIGS["greedy_b1"]
    w = wi.sharpened(wi.make_weights(cfg), 8.0)   # peaked soft-max, as a trained model's; same greedy output
    enc, lens = wi.make_batch(cfg)
    T, K = 250, 4
    model = WindModel.from_config(cfg, w)
    d_enc = torch.from_numpy(enc[0, :T]).cuda()
    res = {"workload": f"greedy_b1 model with its output layer times 8, first {T} frames, beam {K}, S={cfg.S}, "
                       "prefix step 'keep'"}
    for exact in (0, 1):
        model.set_option("beam_exact", exact)
        for N in (1, 16):
            model.beam_decode(d_enc[:32].contiguous(), N, K, cfg.S)
            t0 = time.perf_counter()
            tok, frm, score, st = model.beam_decode(d_enc, N, K, cfg.S)
            sec = time.perf_counter() - t0
            res[f"{'fp32' if exact else 'bf16'}_logits_N{N}"] = {
                "ms": round(sec * 1e3, 2), "frames_per_s": round(T / sec, 1), "passes": int(st.rounds),
                "us_per_pass": round(sec * 1e6 / max(1, st.rounds), 1), "labels": int(len(tok)),
                "decoder_steps": int(st.decoder_steps), "completions": int(st.completions), "score": round(score, 3)}
    model.close()
    return res


def cpu_baseline(wi, cfg, enc, lens, w, budget_frames):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np

    import oracle

    o = oracle.Oracle.from_config(cfg, w)
    threads = min(16, os.cpu_count() or 1, oracle.num_threads())
    # sample: the shortest utterances whose frames add up to about the budget (all of them for B=1)
    order = np.argsort(lens)
    pick, tot = [], 0
    for b in order:
        if pick and tot + lens[b] > budget_frames:
            break
        pick.append(int(b))
        tot += int(lens[b])
    sub_enc = np.ascontiguousarray(enc[pick])
    sub_len = np.ascontiguousarray(lens[pick])
    # the sample is decoded again and again until about ten seconds of CPU work have been timed
    reps, sec = 0, 0.0
    while sec < 10.0 and reps < 64:
        t0 = time.perf_counter()
        o.greedy_batch(sub_enc, sub_len, cfg.S, threads=threads)
        sec += time.perf_counter() - t0
        reps += 1
    used = min(threads, len(pick))
    return {"value": tot * reps / sec, "unit": "frames/s", "cores": used, "kind": "oracle",
            "sample": f"{len(pick)} of {len(lens)} utterances of {cfg.name} ({tot} frames), decoded {reps} times, "
                      f"sequential greedy in fp64, one thread per utterance", "seconds": sec}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="greedy_b1")
    ap.add_argument("--roofline-workload", default="largevocab_b128")
    ap.add_argument("--roofline-window", type=int, default=16)
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true",
                    help="skip the headline workload; used under rocprofv3 --pmc, where every dispatch is serialised")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device copy, the known-size reference for the HBM byte counters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ablation", action="store_true", help="skip the graph / no-graph table at batch 16")
    ap.add_argument("--beam-only", action="store_true", help="only the beam-search figures (for profiling them)")
    ap.add_argument("--print-kernel-digest", action="store_true",
                    help="print the hash of the kernel sources that counter summaries under profiles/ record, and exit")
    args = ap.parse_args()
    if args.print_kernel_digest:
        print(kernel_source_digest())
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU (utterances are independent; more GPUs would "
                 "each decode their own share with no exchange); --gpus must be 1")

    import torch

    import wind_inputs as wi
    from paper_2505_13765_amd import WindModel

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    if args.beam_only:
        print(json.dumps({"beam_scoring": beam_scoring(torch, wi, WindModel, args.steps),
                          "beam_search": beam_search(torch, wi, WindModel)}))
        return
    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.roofline_only:
        rcfg, rmodel, rdev, rframes, rres, _ = run_workload(torch, wi, WindModel, args.roofline_workload,
                                                            [args.roofline_window], 1, 0, with_sequential=False)
        rres.pop("workload_stats")
        roof = roofline_leg(torch, rcfg, rmodel, rdev, args.roofline_window)
        print(json.dumps({"roofline": roof}))
        return

    cfg, model, dev, frames, res, host = run_workload(torch, wi, WindModel, args.workload, None,
                                                      args.steps, args.warmup, with_sequential=True)
    wstats = res.pop("workload_stats")
    best_w = max((k for k in res if k != "seq"), key=lambda k: res[k]["frames_per_s"])
    line = {
        "metric": "encoder frames decoded/sec", "value": res[best_w]["frames_per_s"], "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res[best_w]["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} T~{cfg.len_hi} D={cfg.D} Hj={cfg.Hj} V={cfg.V}+blank "
                               f"L={cfg.L} S={cfg.S}", "window": int(best_w), "frames_per_step": frames},
        "rtfx": res[best_w]["rtfx"], "workload_stats": wstats,
        "sweep": {k: {kk: (round(vv, 3) if isinstance(vv, float) else vv) for kk, vv in v.items()}
                  for k, v in res.items()},
        "speedup_vs_w1": {k: res[k]["frames_per_s"] / res["1"]["frames_per_s"] for k in res if "1" in res},
        "paper_context": "paper: up to 2.4x greedy (W=8/16 vs W=1), 1.26x batched, on 2x A6000, encoder included",
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wi, cfg, host[0], host[1], host[2], budget_frames=1500)
    model.close()
    del dev, model
    torch.cuda.empty_cache()

    if not args.no_ablation:
        line["graph_ablation"] = graph_ablation(torch, wi, WindModel, max(1, min(args.steps, 3)), 1)
        line["beam_scoring"] = beam_scoring(torch, wi, WindModel, args.steps)
        line["beam_search"] = beam_search(torch, wi, WindModel)
    if not args.no_ablation:
        # the two other batched workloads, whole calls (sequential = Algorithm 1, then their windows)
        others = {}
        for name in ("batch32", "lowblank_b256"):
            if name in (args.workload, args.roofline_workload):
                continue
            ocfg, omodel, odev, oframes, ores, _ = run_workload(torch, wi, WindModel, name, None, 2, 1, with_sequential=True)
            ostats = ores.pop("workload_stats")
            others[name] = {"frames_per_call": oframes, "workload_stats": ostats,
                            "ms_per_step": {k: round(v["ms_per_step"], 3) for k, v in ores.items()},
                            "frames_per_s": {k: round(v["frames_per_s"], 1) for k, v in ores.items()}}
            omodel.close()
            del odev, omodel
            torch.cuda.empty_cache()
        line["other_workloads"] = others
    if not args.no_roofline:
        rcfg, rmodel, rdev, rframes, rres, _ = run_workload(torch, wi, WindModel, args.roofline_workload, None,
                                                            max(1, min(args.steps, 3)), 1, with_sequential=False)
        rstats = rres.pop("workload_stats")
        roof = roofline_leg(torch, rcfg, rmodel, rdev, args.roofline_window)
        roof["workload_stats"] = rstats
        roof["cold_first_call_ms"] = round(next(iter(rres.values())).get("cold_first_call_ms", 0.0), 3)
        roof["frames_per_s"] = {k: round(v["frames_per_s"], 1) for k, v in rres.items()}
        roof["ms_per_step"] = {k: round(v["ms_per_step"], 3) for k, v in rres.items()}
        line["roofline"] = roof
        if not args.no_ablation:
            # what the two shortenings of the per-iteration kernel chain are worth on this workload
            # (options "lstm_rec" and "atomic_lists"), whole calls at the roofline window
            abl = {}
            for key, opts in (("default", {}), ("whole_lstm_steps", {"lstm_rec": 0}), ("compacted_lists", {"atomic_lists": 0}),
                              ("both_off", {"lstm_rec": 0, "atomic_lists": 0})):
                for k, v in {"lstm_rec": 1, "atomic_lists": 1, **opts}.items():
                    rmodel.set_option(k, v)
                sec = timed_decodes(torch, rmodel, rdev[0], rdev[1], args.roofline_window, rcfg.S, 2, 1, rdev[2])
                abl[key] = round(sec * 1e3, 3)
            rmodel.set_option("lstm_rec", 1)
            rmodel.set_option("atomic_lists", 1)
            line["chain_ablation"] = {"workload": f"{rcfg.name} W={args.roofline_window}", "unit": "ms per decode call", **abl}
        rmodel.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
