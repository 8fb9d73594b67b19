"""Offline-profiler sweep on one GPU: step latency over (live batch, context length) for a shard shape.

    python -m paper_2605_23945_amd.profile_grid --config 7b_tp4 [--plan | --batch 1,2,4,... --kv-len 512,2048,8192]
                                                 [--t-cap 1048576] [--l-max 131072] [--steps 60] [--warmup 3] [--reps 5]
                                                 [--layers N]

--plan takes the batch sizes and context lengths of the offline profiler's sampling plan (pat_profile_plan: ten
batch sizes in [1, 256], lengths from 8 to --l-max with a denser ladder below 512, pruned by batch * length <= t_cap)
for the configuration's TP degree.

Prints one JSON line per grid point (the rows the latency predictor consumes): tp_degree, batch, kv_len,
sum_context T, mean/min/std latency in microseconds, tokens/s, algorithmic bytes, fraction of 8 TB/s;
`skipped` = 1 where batch * kv_len exceeds the active-token budget, 2 where the point does not fit the pool.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import pat_inputs as pi
    import paper_2605_23945_amd as pat

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="7b_tp4")
    ap.add_argument("--batch", default="")
    ap.add_argument("--kv-len", default="")
    ap.add_argument("--plan", action="store_true", help="the offline profiler's sampling plan instead of --batch/--kv-len")
    ap.add_argument("--l-max", type=int, default=128 * 1024, help="longest context of the plan")
    ap.add_argument("--t-cap", type=int, default=0, help="active-token budget; 0 = what fits in 200 GiB of KV pool")
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0, help="reduced depth (0 = the configuration's)")
    ap.add_argument("--preheat-seconds", type=float, default=30.0,
                    help="decode steps run before the first point, so that every point sees the GPU under sustained load")
    args = ap.parse_args()
    conf = pi.CONFIGS[args.config]
    shard = conf["shard"].with_layers(args.layers) if args.layers else conf["shard"]
    Bs = [int(x) for x in args.batch.split(",")] if args.batch else list(conf.get("grid_b", (1, 2, 4, 8, 16, 32, 64, 128, 256)))
    Ls = [int(x) for x in args.kv_len.split(",")] if args.kv_len else list(conf.get("grid_l", (512, 2048, 8192)))
    kv_bytes_per_token = shard.n_layers * 2 * shard.hkv * shard.head_dim * 2
    t_cap = args.t_cap
    if t_cap <= 0:
        t_cap = 1 << 10
        while (t_cap * 2) * kv_bytes_per_token <= 200 * (1 << 30) and t_cap < (1 << 22):
            t_cap *= 2
    if args.plan:
        pts = [(b, l) for tp, b, l in pat.pat_profile_plan(shard.tp, t_cap, min(args.l_max, t_cap)) if tp == shard.tp]
        Bs = sorted({b for b, _ in pts})
        Ls = sorted({l for _, l in pts})
    extra = args.warmup + args.steps + 2
    cfg = pat.make_cfg(shard, max(Bs), max(Ls) + extra + 64, t_cap + (extra + 64) * max(Bs), 64)
    dec = pat.Decoder(cfg)
    pat.load_synthetic_weights(dec, shard)
    print(json.dumps({"config": args.config, "tp_degree": shard.tp, "n_layers": shard.n_layers, "t_cap": t_cap,
                      "steps": args.steps, "warmup": args.warmup, "reps": args.reps, "plan": bool(args.plan), "preheat_seconds": args.preheat_seconds,
                      "batches": Bs, "kv_lens": Ls}), flush=True)
    import time
    t0 = time.time()
    while time.time() - t0 < args.preheat_seconds:
        dec.pat_profile_grid([min(16, max(Bs))], [min(2048, max(Ls))], t_cap, steps=60, warmup=0, reps=1)
    for b in Bs:                      # one call per batch size so that rows stream out as they are measured
        ls_b = [l for l in Ls if b * l <= t_cap] if args.plan else Ls
        for r in dec.pat_profile_grid([b], ls_b, t_cap, steps=args.steps, warmup=args.warmup, reps=args.reps):
            print(json.dumps({k: (round(v, 3) if isinstance(v, float) else v) for k, v in r.items()}), flush=True)
    dec.close()


if __name__ == "__main__":
    main()
