"""Long-tail rollout of any workload configuration on one GPU, with admission under a KV budget.

    python -m paper_2605_23945_amd.rollout --config 13b_tp2 [--max-live 256] [--kv-gib 160] [--layers N]
                                           [--prompts N] [--max-steps N]

The configuration's prompts wait in a queue; a request is admitted (in request order) when a batch
slot is free and its whole life (prompt + response length) fits the KV-token budget next to the
requests already running: the paper's active-token budget "determined by the runtime KV cache
capacity" (Sec. 4.1), applied at admission so that no step can run out of pages.  Finished sequences
leave by on-device compaction after every step that finished one; admissions happen between steps and
are not timed (their cost here is the generation of synthetic K/V prefixes).  Prints one JSON object:
tokens/s over the timed decode steps and step latency / fraction of 8 TB/s by live batch.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

HBM_PEAK = 8.0e12


def main():
    import numpy as np
    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="13b_tp2")
    ap.add_argument("--max-live", type=int, default=256)
    ap.add_argument("--kv-gib", type=float, default=160.0, help="size of the paged KV pool")
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--prompts", type=int, default=0, help="first N requests only (0 = all)")
    ap.add_argument("--max-steps", type=int, default=0)
    args = ap.parse_args()
    conf = pi.CONFIGS[args.config]
    shard = conf["shard"].with_layers(args.layers) if args.layers else conf["shard"]
    req = pi.rollout_requests(shard, conf["n_prompts"], conf["prompt_len"], resp=conf.get("resp"), steps=conf.get("steps"))
    n = len(req["seq_id"]) if args.prompts <= 0 else min(args.prompts, len(req["seq_id"]))
    need = (req["kv_len"].astype(np.int64) + req["target"])[:n]
    kv_bytes_per_token = shard.n_layers * 2 * shard.hkv * shard.head_dim * 2
    budget = int(args.kv_gib * (1 << 30) // kv_bytes_per_token)
    max_live = min(args.max_live, n)
    if int(need.max()) + 64 > budget:
        raise SystemExit("the longest request does not fit the KV pool")
    dev = "cuda:0"
    dec = pat.Decoder(pat.make_cfg(shard, max_live, int(need.max()) + 1, budget + 64 * max_live, 64), dev)
    pat.load_synthetic_weights(dec, shard, dev)

    waiting = list(range(n))
    running_need = []                  # reserved tokens of the live slots, in slot order
    target_left = []                   # steps each live slot still runs

    def admit():
        batch = []
        while waiting and len(running_need) + len(batch) < max_live and \
                sum(running_need) + sum(int(need[i]) for i in batch) + int(need[waiting[0]]) <= budget:
            batch.append(waiting.pop(0))
        if batch:
            print(f"admitting {len(batch)} requests", file=sys.stderr, flush=True)
            pat.admit_synthetic(dec, shard, req, dev, idx=batch)
            running_need.extend(int(need[i]) for i in batch)
            target_left.extend(int(req["target"][i]) for i in batch)
        return len(batch)

    admit()
    torch.cuda.synchronize()
    lives, ms, wbytes, kvbytes = [], [], [], []
    tokens = 0
    pending = []                       # (events, live) of steps whose time has not been read yet
    steps = 0
    while running_need and (args.max_steps <= 0 or steps < args.max_steps):
        live = len(running_need)
        wb, kb = dec.pat_step_algo_bytes()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dec.pat_decode_step(report=False)
        new_live = dec.pat_kv_compact()
        b.record()
        pending.append((a, b))
        lives.append(live); wbytes.append(wb); kvbytes.append(kb)
        tokens += live
        steps += 1
        target_left[:] = [t - 1 for t in target_left]
        keep = [j for j, t in enumerate(target_left) if t > 0]
        assert len(keep) == new_live
        running_need[:] = [running_need[j] for j in keep]
        target_left[:] = [target_left[j] for j in keep]
        if waiting and len(keep) < live:
            torch.cuda.synchronize()
            admit()
            torch.cuda.synchronize()
        if len(pending) >= 512:
            torch.cuda.synchronize()
            ms += [x.elapsed_time(y) for x, y in pending]; pending.clear()
            print(f"step {steps}: live {len(running_need)}, waiting {len(waiting)}, {sum(ms) * 1e-3:.1f} s in steps", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    ms += [x.elapsed_time(y) for x, y in pending]
    ms = np.array(ms); lives = np.array(lives); byt = np.array(wbytes) + np.array(kvbytes)
    table = []
    for lo, hi in ((1, 1), (2, 2), (3, 4), (5, 8), (9, 16), (17, 32), (33, 64), (65, 128), (129, 256), (257, 1024)):
        sel = (lives >= lo) & (lives <= hi)
        if sel.any():
            table.append({"batch": f"{lo}-{hi}" if lo != hi else str(lo), "steps": int(sel.sum()),
                          "mean_us": round(float(ms[sel].mean() * 1e3), 1),
                          "tokens_per_s": round(float(lives[sel].sum() / (ms[sel].sum() * 1e-3)), 1),
                          "hbm_frac": round(float(byt[sel].sum() / (ms[sel].sum() * 1e-3) / HBM_PEAK), 4)})
    small = lives <= 16
    print(json.dumps({"config": args.config, "tp_degree": shard.tp, "n_layers": shard.n_layers, "requests": n,
                      "max_live": max_live, "kv_token_budget": budget, "steps": int(steps), "tokens": int(tokens),
                      "gpu_seconds_in_steps": round(float(ms.sum()) * 1e-3, 3),
                      "tokens_per_s": round(float(tokens / (ms.sum() * 1e-3)), 2),
                      "hbm_frac_rollout": round(float(byt.sum() / (ms.sum() * 1e-3) / HBM_PEAK), 4),
                      "hbm_frac_batch_le_16": round(float(byt[small].sum() / (ms[small].sum() * 1e-3) / HBM_PEAK), 4) if small.any() else None,
                      "waiting_left": len(waiting), "by_batch": table}))
    dec.close()


if __name__ == "__main__":
    main()
