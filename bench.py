"""Benchmark of the decode-step hot path on one MI355X.

Workload (the configuration the metric is quoted on): Llama-style 7B shape as one GPU's TP=1 shard, 32 layers,
bf16 random weights, 256 prompts of length U[128, 1024], response lengths lognormal(6.0, 0.8) capped at 4096:
a greedy rollout in which the live batch drains from 256 to 1.  A "step" is one decode step of the whole live
batch (every kernel of the path, plus on-device compaction whenever a sequence finished).  All inputs are
resident in HBM before the timed region; the cached K/V are pseudo-random bf16 values (latency does not depend
on them).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 7b_tp1] [--step-log FILE]

With --steps K > 0 (the default is 20) the rollout is SAMPLED: for every live-batch bucket (1, 2, 3-4, 5-8, 9-16,
17-32, 33-64, 65-128, 129-256) the request table is advanced on the host to the middle step of the bucket (lengths
are arithmetic on the table), the sequences alive then are admitted at their lengths of that moment, and W warm-up
plus K timed steps run from there.  The rollout figure (`value`) is the rollout's tokens over the sum, over the
buckets, of (steps the rollout spends in the bucket) x (mean measured step time of the bucket).  With --steps 0 the
whole rollout is run and timed step by step.  After that the same K steps are timed at live batch 1 and 16 on the
other shard shapes (7B TP=4, 13B TP=2, 70B TP=8) and the CPU oracle is timed on a bounded sample.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12
BUCKETS = ((1, 1), (2, 2), (3, 4), (5, 8), (9, 16), (17, 32), (33, 64), (65, 128), (129, 256), (257, 1024))


def bucket_name(lo, hi):
    return str(lo) if lo == hi else f"{lo}-{hi}"


def rollout_plan(req):
    """Host arithmetic on the request table: live batch of every rollout step and the peak of live context tokens."""
    p, t = req["kv_len"].astype(np.int64), req["target"].astype(np.int64)
    steps = int(t.max())
    live = np.array([(t > s).sum() for s in range(steps)], np.int64)
    peak = max(int((p[t > s] + s + 1).sum()) for s in range(steps))
    return steps, live, peak


def fill_kv_pool(dec, seed=0x5EED0002):
    """Pseudo-random N(0, 1) bf16 values over the whole paged pool (what a cached context looks like to the kernels)."""
    import torch
    kv = dec._kv[(-dec._kv.data_ptr()) % 256:]
    n = kv.numel() // 2
    g = torch.Generator(device=kv.device).manual_seed(seed)
    view = kv[: 2 * n].view(torch.bfloat16)
    step = 1 << 28
    for i in range(0, n, step):
        view[i:i + step].normal_(0.0, 1.0, generator=g)


def load_weights(dec, shard, dev, keep_host=False):
    import torch
    import pat_inputs as pi
    from oracle import bits
    m = shard.model
    host_layers = []
    for l in range(m.n_layers):
        w = pi.layer_weights(shard, l, device=dev)
        dec.pat_load_layer(l, w)
        torch.cuda.synchronize()
        if keep_host:
            host_layers.append({k: bits(v) for k, v in w.items()})
        del w
    fw = pi.final_weights(shard, device=dev)
    final_host = {k: bits(v) for k, v in fw.items()} if keep_host else None
    fw["embed"] = pi.embedding_table(shard, device=dev)
    dec.pat_load_final(fw)
    torch.cuda.synchronize()
    return host_layers, final_host


def timed_steps(dec, live, n_steps, profile=False):
    """n_steps decode steps (+ compaction) from the current state, one event pair per step on the launch stream.
    Returns per-step (live batch, context tokens T, microseconds, weight bytes, K/V bytes) and the live batch left."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)]
    rows = []
    if profile:
        dec.pat_timing_enable(True)
    ev[0].record()
    done = 0
    for s in range(n_steps):
        if live == 0:
            break
        wb, kb = dec.pat_step_algo_bytes()
        rows.append([live, kb, 0.0, wb, kb])
        dec.pat_decode_step(report=False)
        live = dec.pat_kv_compact()
        ev[s + 1].record()
        done += 1
    torch.cuda.synchronize()
    if profile:
        dec.pat_timing_enable(False)
    for s in range(done):
        rows[s][2] = ev[s].elapsed_time(ev[s + 1]) * 1e3
    return rows, live


def summarize(name, rows):
    us = np.array([r[2] for r in rows]); b = np.array([r[0] for r in rows]); byt = np.array([r[3] + r[4] for r in rows])
    return {"batch": name, "steps": int(len(rows)), "mean_live_batch": round(float(b.mean()), 2),
            "mean_us": round(float(us.mean()), 1), "p50_us": round(float(np.median(us)), 1), "p99_us": round(float(np.percentile(us, 99)), 1),
            "tokens_per_s": round(float(b.sum() / (us.sum() * 1e-6)), 1),
            "hbm_frac": round(float(byt.sum() / (us.sum() * 1e-6) / HBM_PEAK), 4)}


def class_times(dec):
    """Kernel-class totals of the bracketed (profiled) steps: {class: (ms, launches)}."""
    return {k: dec.pat_timing_read(k) for k in (0, 1, 2, 3)}


def roofline_objects(shard, prof_rows, classes, n_prof_steps, fused):
    """The dominant kernels' achieved bandwidth, from HIP events around every launch of the class on the launch stream."""
    m = shard.model
    out = {}
    gu_bytes = 2.0 * 2 * shard.ffn * m.hidden                           # one gate/up launch streams 2 F x H bf16 weights
    ms, n = classes[3]
    if n:
        out["gate_up"] = {"kernel": "gemm_xs_kernel<.., kGemmSwiGLU> / gemm_xb_kernel (gate/up projection, SiLU*mul epilogue)",
                          "bound": "hbm", "achieved": round(gu_bytes * n / (ms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                          "frac": round(gu_bytes * n / (ms * 1e-3) / HBM_PEAK, 4), "traffic": None, "launches": int(n),
                          "avg_launch_us": round(ms * 1e3 / n, 2), "algo_bytes_per_launch": gu_bytes}
    ms, n = classes[1]
    kv_bytes = float(sum(r[4] for r in prof_rows))                       # K and V of every cached token once per layer
    if n:
        out["attention"] = {"kernel": "attn_stream_kernel + attn_merge_kernel (paged split-KV attention)", "bound": "hbm",
                            "achieved": round(kv_bytes / (ms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                            "frac": round(kv_bytes / (ms * 1e-3) / HBM_PEAK, 4), "traffic": None, "launches": int(n),
                            "avg_launch_us": round(ms * 1e3 / n, 2), "algo_bytes_per_launch": round(kv_bytes / n, 1)}
    ms0, n0 = classes[0]
    w_bytes = float(sum(r[3] for r in prof_rows))
    if n0:
        rest = w_bytes - gu_bytes * classes[3][1]
        out["other_projections"] = {"kernel": ("layer_fused_kernel (O, gate/up, down, next QKV per launch)" if fused else
                                               "gemm_xs_kernel / gemm_xb_kernel (QKV, O, down, vocabulary head)"),
                                    "bound": "hbm", "achieved": round(rest / (ms0 * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                                    "frac": round(rest / (ms0 * 1e-3) / HBM_PEAK, 4), "traffic": None, "launches": int(n0),
                                    "avg_launch_us": round(ms0 * 1e3 / n0, 2)}
    out["everything_else"] = {"kernel": "embedding, argmax, bookkeeping (and rmsnorm_pack above 32 rows)", "total_ms": round(classes[2][0], 3),
                              "launches": int(classes[2][1])}
    out["profiled_steps"] = int(n_prof_steps)
    return out


def cpu_baseline(shard, req, host_layers, final_w, n_rows=8):
    """The CPU oracle as it stands on a bounded sample: (i) the tiny configuration in full (32 steps x 8 sequences) on all
    threads and on one, (ii) one full-depth decode step of `n_rows` sequences of the benchmark's workload on all threads."""
    import pat_inputs as pi
    from oracle import Oracle, OracleDecoder, bits
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    gomp = None
    for name in ("libgomp.so.1", "libgomp.so"):
        try:
            gomp = ctypes.CDLL(name); break
        except OSError:
            pass

    def tiny(nthreads):
        if gomp is not None:
            gomp.omp_set_num_threads(nthreads)
        ts = pi.CONFIGS["tiny_tp1"]["shard"]; tm = ts.model
        treq = pi.rollout_requests(ts, 8, (16, 128), steps=32)
        layers = [{k: bits(v) for k, v in pi.layer_weights(ts, l).items()} for l in range(tm.n_layers)]
        fw = {k: bits(v) for k, v in pi.final_weights(ts).items()}
        od = OracleDecoder(Oracle("f64"), (tm.n_layers, tm.hidden, ts.hq, ts.hkv, tm.head_dim, ts.ffn, tm.rms_eps, tm.rope_base),
                           lambda l: layers[l], fw, lambda tok: bits(pi.embedding_rows(ts, [tok]))[0])
        for i in range(8):
            L = int(treq["kv_len"][i])
            kv = [pi.kv_prefix(ts, int(treq["seq_id"][i]), l, L) for l in range(tm.n_layers)]
            od.admit(treq["seq_id"][i], treq["token"][i], L, 33, [bits(a) for a, _ in kv], [bits(b) for _, b in kv], 34)
        t0 = time.perf_counter()
        for _ in range(32):
            od.step()
        return time.perf_counter() - t0

    t_tiny_all = tiny(threads)
    t_tiny_one = tiny(1) if gomp is not None else None
    if gomp is not None:
        gomp.omp_set_num_threads(threads)
    m = shard.model
    order = np.argsort(req["kv_len"])
    rows = [int(order[len(order) // 2 + i]) for i in range(n_rows)]
    od = OracleDecoder(Oracle("f64"), (m.n_layers, m.hidden, shard.hq, shard.hkv, m.head_dim, shard.ffn, m.rms_eps, m.rope_base),
                       lambda l: host_layers[l], final_w, lambda tok: bits(pi.embedding_rows(shard, [tok]))[0])
    for i in rows:
        L = int(req["kv_len"][i])
        kv = [pi.kv_prefix(shard, int(req["seq_id"][i]), l, L) for l in range(m.n_layers)]
        od.admit(req["seq_id"][i], req["token"][i], L, 8, [bits(a) for a, _ in kv], [bits(b) for _, b in kv], 2)
    t0 = time.perf_counter()
    od.step()
    dt = time.perf_counter() - t0
    return {"value": n_rows / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"one full-depth decode step of {n_rows} sequences (median prompt lengths "
                      f"{[int(req['kv_len'][i]) for i in rows]}) of the same workload, float64, {dt:.1f} s on {threads} threads",
            "tiny_config_full": {"what": "configuration 1 in full: 32 greedy steps x 8 sequences (2 layers, hidden 256)",
                                 "seconds_all_threads": round(t_tiny_all, 3), "tokens_per_s_all_threads": round(256 / t_tiny_all, 1),
                                 "seconds_one_thread": None if t_tiny_one is None else round(t_tiny_one, 3),
                                 "tokens_per_s_one_thread": None if t_tiny_one is None else round(256 / t_tiny_one, 1)},
            "host_cores_visible": os.cpu_count()}


def by_shard_block(names, K, W, dev, kv_len=1024):
    """K timed steps at live batch 1 and 16 on other shard shapes: the target regime on every shard."""
    import gc
    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat
    out = []
    for name in names:
        shard = pi.CONFIGS[name]["shard"]
        B_max, L_max = 16, kv_len + K + W + 8
        dec = pat.Decoder(pat.make_cfg(shard, B_max, L_max, B_max * L_max, 64), dev)
        load_weights(dec, shard, dev)
        fill_kv_pool(dec)
        for B in (1, 16):
            dec.pat_decode_reset()
            ids = np.arange(B, dtype=np.int32)
            dec.pat_decode_admit(ids, (ids * 7919 + 11) % shard.model.vocab, np.full(B, kv_len, np.int32), np.full(B, K + W + 2, np.int32))
            timed_steps(dec, B, W)
            rows, _ = timed_steps(dec, B, K)
            r = summarize(str(B), rows)
            r.update({"shard": name, "kv_len": kv_len, "fused_layer_kernel": dec.pat_decode_uses_fused_kernel()})
            out.append(r)
        dec.close()
        del dec
        gc.collect(); torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="timed steps per live-batch bucket (0 = run and time the whole rollout)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="7b_tp1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-shards", action="store_true", help="skip the live batch 1 / 16 block on the other shard shapes")
    ap.add_argument("--profile-steps", type=int, default=8, help="steps per bucket with every kernel class bracketed by events")
    ap.add_argument("--step-log", default="", help="write one JSON line per timed step (step, live batch, T, us, bytes, GB/s)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (a TP shard is a set of shapes held by one GPU; "
              "no collectives are built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat

    dev = "cuda:0"
    torch.cuda.set_device(0)
    conf = pi.CONFIGS[args.config]
    shard = conf["shard"]
    m = shard.model
    req = pi.rollout_requests(shard, conf["n_prompts"], conf["prompt_len"], resp=conf["resp"])
    n = len(req["seq_id"])
    total_steps, live_of_step, peak_tokens = rollout_plan(req)
    budget = peak_tokens + 64 * n
    max_seq = int((req["kv_len"] + req["target"]).max()) + 1
    dec = pat.Decoder(pat.make_cfg(shard, n, max_seq, budget, page_tokens=64), dev)

    t_setup = time.perf_counter()
    want_cpu = not args.no_cpu_baseline
    host_layers, final_host = load_weights(dec, shard, dev, keep_host=want_cpu)
    fill_kv_pool(dec)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    W, K = max(0, args.warmup), max(0, args.steps)
    p_len, tgt = req["kv_len"].astype(np.int64), req["target"].astype(np.int64)
    rollout_tokens = int(live_of_step.sum())
    step_rows, table, prof_rows_small, prof_rows_large = [], [], [], []
    classes_small = classes_large = None
    t_timed0 = time.perf_counter()

    def admit_at(s):
        """The sequences alive at rollout step s, at their lengths of that moment."""
        dec.pat_decode_reset()
        alive = np.nonzero(tgt > s)[0]
        dec.pat_decode_admit(req["seq_id"][alive], req["token"][alive], (p_len[alive] + s).astype(np.int32), (tgt[alive] - s).astype(np.int32))
        return len(alive)

    if K > 0:
        mode = "sampled"
        est_time_us = 0.0
        for lo, hi in BUCKETS:
            steps_in = np.nonzero((live_of_step >= lo) & (live_of_step <= hi))[0]
            if len(steps_in) == 0:
                continue
            s_mid = int(steps_in[len(steps_in) // 2])
            s_mid = min(s_mid, total_steps - 1)
            live = admit_at(s_mid)
            _, live = timed_steps(dec, live, min(W, max(0, total_steps - s_mid - 1)))
            rows, live = timed_steps(dec, live, K)
            if not rows:                                       # the bucket sits at the very end of the rollout
                live = admit_at(s_mid); rows, live = timed_steps(dec, live, K)
            r = summarize(bucket_name(lo, hi), rows)
            r.update({"rollout_steps_in_bucket": int(len(steps_in)), "sampled_at_rollout_step": s_mid})
            table.append(r)
            est_time_us += len(steps_in) * r["mean_us"]
            step_rows += [[s_mid + i] + row for i, row in enumerate(rows)]
            if args.profile_steps > 0 and live > 0:            # a few more steps with every kernel class bracketed by events
                for k in (0, 1, 2, 3):
                    dec.pat_timing_read(k)
                prow, live = timed_steps(dec, live, args.profile_steps, profile=True)
                ct = class_times(dec)
                if hi <= 16:
                    prof_rows_small += prow
                    classes_small = ct if classes_small is None else {k: (classes_small[k][0] + ct[k][0], classes_small[k][1] + ct[k][1]) for k in ct}
                elif lo >= 129:
                    prof_rows_large += prow
                    classes_large = ct
        value = rollout_tokens / (est_time_us * 1e-6)
        ms_per_step = est_time_us * 1e-3 / total_steps
        timed_total = sum(r["steps"] for r in table)
    else:
        mode = "full"
        live = admit_at(0)
        _, live = timed_steps(dec, live, W)
        rows, live = timed_steps(dec, live, total_steps - W)
        step_rows = [[W + i] + row for i, row in enumerate(rows)]
        lives = np.array([r[0] for r in rows])
        for lo, hi in BUCKETS:
            sel = [r for r in rows if lo <= r[0] <= hi]
            if sel:
                table.append(summarize(bucket_name(lo, hi), sel))
        us_total = sum(r[2] for r in rows)
        value = float(lives.sum()) / (us_total * 1e-6)
        ms_per_step = us_total * 1e-3 / len(rows)
        timed_total = len(rows)
    gpu_wall = time.perf_counter() - t_timed0

    small = [r for r in step_rows if r[1] <= 16]
    frac_small = (sum(r[4] + r[5] for r in small) / (sum(r[3] for r in small) * 1e-6) / HBM_PEAK) if small else None
    if K > 0 and table:                                         # weighted by the rollout's step histogram, like `value`
        num = sum(t["rollout_steps_in_bucket"] * t["mean_us"] * t["hbm_frac"] for t in table if int(t["batch"].split("-")[-1]) <= 16)
        den = sum(t["rollout_steps_in_bucket"] * t["mean_us"] for t in table if int(t["batch"].split("-")[-1]) <= 16)
        frac_small = num / den if den else frac_small
    all_bytes = sum(r[4] + r[5] for r in step_rows); all_us = sum(r[3] for r in step_rows)

    fused = dec.pat_decode_uses_fused_kernel()
    regimes = {}
    if classes_small is not None:
        regimes["live_batch_le_16"] = roofline_objects(shard, prof_rows_small, classes_small, len(prof_rows_small), fused)
    if classes_large is not None:
        regimes["live_batch_ge_129"] = roofline_objects(shard, prof_rows_large, classes_large, len(prof_rows_large), False)
    roof = None
    if "live_batch_le_16" in regimes and "gate_up" in regimes["live_batch_le_16"]:
        roof = dict(regimes["live_batch_le_16"]["gate_up"])
        roof["regime"] = "live batch <= 16 (the target regime): the gate/up projection is the kernel with the largest share of the step"
    elif "live_batch_ge_129" in regimes:
        roof = dict(regimes["live_batch_ge_129"]["attention"]); roof["regime"] = "live batch >= 129"
    if roof is not None:
        roof["by_regime"] = regimes

    if args.step_log:
        with open(args.step_log, "w") as f:
            for s, b, t_ctx, us, wb, kb in step_rows:
                f.write(json.dumps({"rollout_step": int(s), "live_batch": int(b), "kv_bytes": kb, "us": round(us, 2),
                                    "algo_bytes": wb + kb, "GBps": round((wb + kb) / (us * 1e-6) / 1e9, 1)}) + "\n")

    dec.close()
    del dec
    torch.cuda.empty_cache()
    shards = None if args.no_shards or K == 0 else by_shard_block([c for c in ("7b_tp4", "13b_tp2", "70b_tp8") if c != args.config], K, W, dev)
    cpu = cpu_baseline(shard, req, host_layers, final_host) if want_cpu else None

    out = {
        "metric": ("decode tokens/s over the long-tail rollout, live batch 256 -> 1 (per-batch step latency and %HBM in by_batch)"
                   + ("; rollout figure assembled from K timed steps at the middle of every live-batch bucket, weighted by the "
                      "rollout's step histogram" if mode == "sampled" else "; whole rollout timed")),
        "value": round(value, 2), "unit": "tokens/s", "n_gpus": 1, "steps": int(K if K > 0 else timed_total), "warmup": int(W),
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: {m.n_layers} layers, hidden {m.hidden}, {shard.hq} q / {shard.hkv} kv heads x "
                               f"{m.head_dim}, FFN {shard.ffn}, vocab slice {shard.vocab}; {n} prompts U{list(conf['prompt_len'])}, "
                               f"lognormal{list(conf['resp'])} responses; live batch {n}->1",
                   "tp_degree": shard.tp, "rollout_steps": total_steps, "rollout_tokens": rollout_tokens,
                   "peak_context_tokens": peak_tokens, "page_tokens": 64, "mode": mode,
                   "fused_layer_kernel_at_batch_le_16": fused},
        "timed_steps_total": int(timed_total), "timed_region_wall_seconds": round(gpu_wall, 3), "setup_seconds": round(t_setup, 1),
        "hbm_frac_timed_steps": round(float(all_bytes / (all_us * 1e-6) / HBM_PEAK), 4),
        "hbm_frac_batch_le_16": None if frac_small is None else round(float(frac_small), 4),
        "by_batch": table,
        "by_shard": shards,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
