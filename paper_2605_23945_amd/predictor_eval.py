"""Accuracy of the latency predictor on this GPU: fit on a sparse profile grid, check on points and
on a rollout the fit has not seen.

    python -m paper_2605_23945_amd.predictor_eval [--config 7b_tp1] [--layers N] [--t-cap 262144]
        [--fit-batch 1,4,16,64,256] [--fit-len 256,1024,4096] [--test-batch 2,8,32,128] [--test-len 512,2048]
        [--rollout-prompts 96] [--steps 30] [--reps 2] [--plan [--l-max 16384]]

--plan fits on the offline profiler's sampling plan for the shard's TP degree (pat_profile_plan: ten batch sizes,
lengths from 8 to --l-max, two per octave below 512, pruned by batch * length <= t_cap) instead of --fit-batch x
--fit-len; the held-out points then default to batch sizes and lengths between the plan's, half of them below 512.

1. Profile grid over the fit points (the offline profiler's protocol), predictor fitted to it.
2. The same protocol at held-out (batch, length) points: predicted vs measured step latency.
3. A synthetic long-tail rollout of the configuration (fewer prompts): every decode step's measured
   latency against the prediction for that step's (live batch, context tokens), the way the switch
   controller would query it.
Prints one JSON object: per-point errors and mean / max absolute relative error of 2 and 3.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import numpy as np
    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="7b_tp1")
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--t-cap", type=int, default=1 << 18)
    ap.add_argument("--fit-batch", default="1,4,16,64,256")
    ap.add_argument("--fit-len", default="256,1024,4096")
    ap.add_argument("--test-batch", default="2,8,32,128")
    ap.add_argument("--test-len", default="512,2048")
    ap.add_argument("--rollout-prompts", type=int, default=96)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--reps", type=int, default=2)
    ap.add_argument("--preheat-seconds", type=float, default=30.0,
                    help="decode steps run before anything is measured: under sustained load the step of the widest "
                         "shards is about 5 %% slower than on a GPU that has just started, and generation is sustained load")
    ap.add_argument("--plan", action="store_true")
    ap.add_argument("--l-max", type=int, default=16384)
    args = ap.parse_args()
    ints = lambda s: [int(x) for x in s.split(",") if x]
    conf = pi.CONFIGS[args.config]
    shard = conf["shard"].with_layers(args.layers) if args.layers else conf["shard"]
    fit_b, fit_l, test_b, test_l = ints(args.fit_batch), ints(args.fit_len), ints(args.test_batch), ints(args.test_len)
    if args.plan:
        pts = [(b, l) for tp, b, l in pat.pat_profile_plan(shard.tp, args.t_cap, min(args.l_max, args.t_cap)) if tp == shard.tp]
        fit_b, fit_l = sorted({b for b, _ in pts}), sorted({l for _, l in pts})
        if args.test_batch == ap.get_default("test_batch"):
            test_b = [3, 12, 48, 160]
        if args.test_len == ap.get_default("test_len"):
            test_l = [20, 80, 320, 1536, 6000]

    n_roll = args.rollout_prompts
    req = pi.rollout_requests(shard, n_roll, conf["prompt_len"], resp=conf["resp"]) if n_roll > 0 else None
    extra = 3 + args.steps + 1
    max_b = max(fit_b + test_b + [n_roll])
    max_seq = max(fit_l + test_l) + extra + 64
    budget = args.t_cap + (extra + 64) * max_b
    if req is not None:
        max_seq = max(max_seq, int((req["kv_len"] + req["target"]).max()) + 1)
        budget = max(budget, int((req["kv_len"] + req["target"]).sum()) + 64 * n_roll)
    dec = pat.Decoder(pat.make_cfg(shard, max_b, max_seq, budget, 64))
    pat.load_synthetic_weights(dec, shard)

    def grid(bs, ls):
        rows = []
        for b in bs:
            rows += [r for r in dec.pat_profile_grid([b], ls, args.t_cap, steps=args.steps, warmup=3, reps=args.reps)
                     if r["skipped"] == 0]
            print(f"profiled batch {b}: {len(rows)} points so far", file=sys.stderr, flush=True)
        return rows

    import time
    t0 = time.time()
    while time.time() - t0 < args.preheat_seconds:
        dec.pat_profile_grid([min(16, max_b)], [min(2048, max(fit_l))], args.t_cap, steps=60, warmup=0, reps=1)
    print(f"preheated for {time.time() - t0:.0f} s", file=sys.stderr, flush=True)
    fit_rows = grid(fit_b, fit_l)
    pred = pat.Predictor([(r["tp_degree"], r["batch"], r["sum_context"], r["mean_us"]) for r in fit_rows])
    held = []
    for r in grid(test_b, test_l):
        p = pred.pat_predictor_query(r["tp_degree"], r["batch"], r["sum_context"])
        held.append({"batch": r["batch"], "kv_len": r["kv_len"], "measured_us": round(r["mean_us"], 1),
                     "predicted_us": round(p, 1), "rel_err": round(p / r["mean_us"] - 1.0, 4)})
    lines = []
    for b in fit_b:
        al, be = pred.pat_predictor_line(shard.tp, b)
        res = [(r["kv_len"], (al + be * r["sum_context"]) / r["mean_us"] - 1.0) for r in fit_rows if r["batch"] == b]
        lines.append({"batch": b, "alpha_us": round(al, 1), "beta_us_per_token": round(be, 6), "points": len(res),
                      "max_abs_residual_below_512": round(max([abs(e) for l, e in res if l < 512], default=0.0), 4),
                      "max_abs_residual_from_512": round(max([abs(e) for l, e in res if l >= 512], default=0.0), 4)})
    out = {"config": args.config, "tp_degree": shard.tp, "n_layers": shard.n_layers, "plan": bool(args.plan),
           "preheat_seconds": args.preheat_seconds,
           "fit_batches": fit_b, "fit_lengths": fit_l, "lines": lines,
           "fit_points": len(fit_rows), "held_out": held,
           "held_out_mean_abs_err": round(float(np.mean([abs(h["rel_err"]) for h in held])), 4) if held else None,
           "held_out_max_abs_err": round(float(np.max([abs(h["rel_err"]) for h in held])), 4) if held else None}

    if req is not None:
        dec.pat_decode_reset()
        pat.admit_synthetic(dec, shard, req, "cuda:0")
        live = n_roll
        ctx = req["kv_len"].astype(np.int64).copy()
        gen = np.zeros(n_roll, np.int64)
        tgt = req["target"].astype(np.int64)
        alive = np.ones(n_roll, bool)
        total = int(tgt.max())
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(total + 1)]
        Bs, Ts = [], []
        torch.cuda.synchronize()
        ev[0].record()
        for s in range(total):
            Bs.append(live); Ts.append(int(ctx[alive].sum()))          # what the executor reports before the step
            dec.pat_decode_step(report=False)
            live = dec.pat_kv_compact()
            ev[s + 1].record()
            ctx[alive] += 1; gen[alive] += 1
            alive &= gen < tgt
            assert live == int(alive.sum())
        torch.cuda.synchronize()
        ms = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(total)]) * 1e3
        pr = np.array([pred.pat_predictor_query(shard.tp, b, t) for b, t in zip(Bs, Ts)])
        rel = pr / ms - 1.0
        Bs = np.array(Bs)
        buckets = []
        for lo, hi in ((1, 1), (2, 4), (5, 16), (17, 64), (65, 256)):
            m = (Bs >= lo) & (Bs <= hi)
            if m.any():
                buckets.append({"batch": f"{lo}-{hi}", "steps": int(m.sum()), "mean_abs_err": round(float(np.abs(rel[m]).mean()), 4),
                                "bias": round(float(rel[m].mean()), 4)})
        out["rollout"] = {"prompts": n_roll, "steps": total, "measured_total_ms": round(float(ms.sum()) / 1e3, 2),
                          "predicted_total_ms": round(float(pr.sum()) / 1e3, 2),
                          "mean_abs_err": round(float(np.abs(rel).mean()), 4), "p95_abs_err": round(float(np.percentile(np.abs(rel), 95)), 4),
                          "by_batch": buckets}
    dec.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
