"""Benchmark of the decode-step hot path on one MI355X.

Workload (the configuration the metric is quoted on): Llama-style 7B shape as one GPU's
TP=1 shard, 32 layers, bf16 random weights, 256 prompts of length U[128, 1024], response
lengths lognormal(6.0, 0.8) capped at 4096: a full greedy rollout in which the live batch
drains from 256 to 1.  A "step" is one decode step of the whole live batch (every kernel of
the path, plus on-device compaction whenever a sequence finished).  All inputs are resident
in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 7b_tp1]

Without --steps the whole rollout after the warm-up steps is timed.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12


def plan_rollout(req):
    """Host arithmetic on the request lengths: number of steps and the peak of live context tokens."""
    p, t = req["kv_len"].astype(np.int64), req["target"].astype(np.int64)
    steps = int(t.max())
    peak = 0
    for s in range(steps):
        live = t > s
        peak = max(peak, int((p[live] + s + 1).sum()))
    return steps, peak


def cpu_baseline(shard, req, host_layers, final_w, n_rows=8):
    """Times the CPU oracle (as it stands) on a bounded sample: one full-depth decode step of
    `n_rows` sequences of the workload (those with the median prompt lengths)."""
    import pat_inputs as pi
    from oracle import Oracle, OracleDecoder, bits
    m = shard.model
    order = np.argsort(req["kv_len"])
    rows = [int(order[len(order) // 2 + i]) for i in range(n_rows)]
    emb = lambda tok: bits(pi.embedding_rows(shard, [tok]))[0]
    od = OracleDecoder(Oracle("f64"), (m.n_layers, m.hidden, shard.hq, shard.hkv, m.head_dim, shard.ffn, m.rms_eps,
                                       m.rope_base), lambda l: host_layers[l], final_w, emb)
    for i in rows:
        L = int(req["kv_len"][i])
        kv = [pi.kv_prefix(shard, int(req["seq_id"][i]), l, L) for l in range(m.n_layers)]
        od.admit(req["seq_id"][i], req["token"][i], L, 8, [bits(a) for a, _ in kv], [bits(b) for _, b in kv], 2)
    t0 = time.perf_counter()
    od.step()
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n_rows / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"one full-depth decode step of {n_rows} sequences (median prompt lengths "
                      f"{[int(req['kv_len'][i]) for i in rows]}) of the same workload, float64, {dt:.1f} s",
            "host_cores_visible": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0 = the whole rollout)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="7b_tp1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-every", type=int, default=32, help="bracket kernels with events every N-th step")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (a TP shard is a set of shapes held by one GPU; "
              "no collectives are built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat
    from oracle import bits

    dev = "cuda:0"
    torch.cuda.set_device(0)
    conf = pi.CONFIGS[args.config]
    shard = conf["shard"]
    m = shard.model
    req = pi.rollout_requests(shard, conf["n_prompts"], conf["prompt_len"], resp=conf["resp"])
    n = len(req["seq_id"])
    total_steps, peak_tokens = plan_rollout(req)
    budget = peak_tokens + 64 * n
    max_seq = int((req["kv_len"] + req["target"]).max()) + 1
    cfg = pat.make_cfg(shard, n, max_seq, budget, page_tokens=64)
    dec = pat.Decoder(cfg, dev)

    t_setup = time.perf_counter()
    want_cpu = not args.no_cpu_baseline
    host_layers = []
    for l in range(m.n_layers):
        w = pi.layer_weights(shard, l, device=dev)
        dec.pat_load_layer(l, w)
        torch.cuda.synchronize()
        if want_cpu:
            host_layers.append({k: bits(v) for k, v in w.items()})
        del w
    fw = pi.final_weights(shard, device=dev)
    final_host = {k: bits(v) for k, v in fw.items()} if want_cpu else None
    fw["embed"] = pi.embedding_table(shard, device=dev)
    dec.pat_load_final(fw)
    torch.cuda.synchronize()
    del fw
    pat.admit_synthetic(dec, shard, req, dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    W = max(0, args.warmup)
    K = args.steps if args.steps > 0 else total_steps - W
    K = min(K, total_steps - W)
    live = n
    lives, tokens = [], 0
    for _ in range(W):
        dec.pat_decode_step(report=False)
        live = dec.pat_kv_compact()

    events = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    wbytes, kvbytes, prof_steps = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events[0].record()
    for s in range(K):
        wb, kb = dec.pat_step_algo_bytes()
        wbytes.append(wb); kvbytes.append(kb); lives.append(live)
        prof = args.profile_every > 0 and s % args.profile_every == 0
        if prof:
            dec.pat_timing_enable(True)
        dec.pat_decode_step(report=False)
        if prof:
            dec.pat_timing_enable(False)          # drains the stream and adds this step's kernel times
            prof_steps.append(s)
        tokens += live
        live = dec.pat_kv_compact()
        events[s + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_ms = np.array([events[i].elapsed_time(events[i + 1]) for i in range(K)])
    gpu_s = float(events[0].elapsed_time(events[K])) * 1e-3
    lives = np.array(lives); wbytes = np.array(wbytes); kvbytes = np.array(kvbytes)

    # latency / tokens/s / %HBM per live-batch bucket (profiled steps carry event overhead: left out)
    clean = np.ones(K, bool); clean[prof_steps] = False
    table = []
    for lo, hi in ((1, 1), (2, 2), (3, 4), (5, 8), (9, 16), (17, 32), (33, 64), (65, 128), (129, 256), (257, 1024)):
        sel = (lives >= lo) & (lives <= hi) & clean
        if sel.any():
            us = step_ms[sel] * 1e3
            byt = (wbytes[sel] + kvbytes[sel])
            table.append({"batch": f"{lo}-{hi}" if lo != hi else str(lo), "steps": int(sel.sum()),
                          "mean_us": round(float(us.mean()), 1), "p50_us": round(float(np.median(us)), 1),
                          "p99_us": round(float(np.percentile(us, 99)), 1),
                          "tokens_per_s": round(float(lives[sel].sum() / (us.sum() * 1e-6)), 1),
                          "hbm_frac": round(float(byt.sum() / (us.sum() * 1e-6) / HBM_PEAK), 4)})
    small = (lives <= 16) & clean
    frac_small = float((wbytes[small] + kvbytes[small]).sum() / (step_ms[small].sum() * 1e-3) / HBM_PEAK) if small.any() else None

    # dominant kernel class, measured live with HIP events on the step's stream
    t_gemm, n_gemm = dec.pat_timing_read(0)
    t_attn, n_attn = dec.pat_timing_read(1)
    t_misc, n_misc = dec.pat_timing_read(2)
    ps = np.array(prof_steps, int)
    roof = None
    if len(ps) and n_gemm:
        gemm_b, attn_b = float(wbytes[ps].sum()), float(kvbytes[ps].sum())
        cand = {"gemm_xs_kernel / gemm_xb_kernel (+ gemm_reduce_kernel): weight-streaming projections": (gemm_b, t_gemm, n_gemm),
                "attn_stream_kernel + attn_merge_kernel (paged split-KV attention)": (attn_b, t_attn, n_attn)}
        name = max(cand, key=lambda k: cand[k][1])
        def obj(k):
            b, t, cnt = cand[k]
            return {"kernel": k, "bound": "hbm", "achieved": round(b / (t * 1e-3) / 1e9, 1), "peak": 8000.0,
                    "unit": "GB/s", "frac": round(b / (t * 1e-3) / HBM_PEAK, 4), "traffic": None,
                    "launches": int(cnt), "avg_launch_us": round(t * 1e3 / cnt, 2),
                    "algo_bytes_per_launch": round(b / cnt, 1)}
        roof = obj(name)
        other = [k for k in cand if k != name][0]
        roof["other_classes"] = [obj(other), {"kernel": "norm/rope/argmax/bookkeeping", "total_ms": round(t_misc, 3),
                                               "launches": int(n_misc)}]
        roof["sampled_steps"] = int(len(ps))

    cpu = None
    if want_cpu:
        cpu = cpu_baseline(shard, req, host_layers, final_host)

    out = {
        "metric": "decode tokens/s over the long-tail rollout (per-batch step latency and %HBM in by_batch)",
        "value": round(tokens / gpu_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": int(K), "warmup": int(W),
        "ms_per_step": round(gpu_s * 1e3 / K, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: {m.n_layers} layers, hidden {m.hidden}, {shard.hq} q / {shard.hkv} kv heads x "
                               f"{m.head_dim}, FFN {shard.ffn}, vocab slice {shard.vocab}; {n} prompts U{list(conf['prompt_len'])}, "
                               f"lognormal{list(conf['resp'])} responses; live batch {n}->1",
                   "tp_degree": shard.tp, "rollout_steps": total_steps, "peak_context_tokens": peak_tokens,
                   "page_tokens": 64},
        "tokens": int(tokens), "gpu_seconds": round(gpu_s, 3), "host_wall_seconds": round(wall, 3),
        "setup_seconds": round(t_setup, 1),
        "hbm_frac_rollout": round(float((wbytes.sum() + kvbytes.sum()) / gpu_s / HBM_PEAK), 4),
        "hbm_frac_batch_le_16": None if frac_small is None else round(frac_small, 4),
        "by_batch": table,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
