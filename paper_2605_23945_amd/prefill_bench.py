"""Prefill latency table of a shard on this GPU: the T_prefill(TP, batch, length) samples that the
recomputation estimate of the switch decision interpolates (Eq. (4)).

    python -m paper_2605_23945_amd.prefill_bench [--config 7b_tp1] [--layers N] [--batch 1,4,16] [--len 256,1024,4096]
                                                 [--pass-width 256] [--reps 2]

Calls pat_profile_prefill: for each (batch, length) it admits `batch` sequences of `length` positions (page
contents are whatever the pool holds; the prefill overwrites them), rebuilds their K/V from seeded token ids
with pat_prefill and times the call with HIP events on the launch stream (the call waits for the GPU after
every pass, so the host time between passes is inside the figure).  Prints one JSON object; `rows` holds the table in
the layout of pat_prefill_row.  flops = 2 x projection weights x tokens + the causal attention's
4 x hq x d x length^2 / 2 per sequence and layer; the fraction is against the dense bf16 MFMA peak.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

MFMA_BF16_PEAK = 2.5e15


def main():
    import numpy as np
    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="7b_tp1")
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--batch", default="1,4,16")
    ap.add_argument("--len", default="256,1024,4096")
    ap.add_argument("--pass-width", type=int, default=256)
    ap.add_argument("--reps", type=int, default=2)
    args = ap.parse_args()
    ints = lambda s: [int(x) for x in s.split(",") if x]
    conf = pi.CONFIGS[args.config]
    shard = conf["shard"].with_layers(args.layers) if args.layers else conf["shard"]
    bs, ls = ints(args.batch), ints(args.len)
    width = max(args.pass_width, max(bs))
    dec = pat.Decoder(pat.make_cfg(shard, width, max(ls) + 8, max(bs) * max(ls) + 64 * max(bs), 64))
    pat.load_synthetic_weights(dec, shard)
    m = shard.model
    per_tok = 2.0 * shard.n_layers * (shard.hidden * (shard.hq + 2 * shard.hkv) * m.head_dim + shard.hidden * shard.hq * m.head_dim
                                      + 3 * shard.hidden * shard.ffn)
    _, prof = dec.pat_profile_prefill(bs, ls, 1 << 40, reps=args.reps)
    rows = []
    for r in prof:
        b, L, us = r["batch"], r["length"], r["latency_us"]
        if us < 0:
            rows.append({"tp_degree": shard.tp, "batch": b, "length": L, "latency_us": None})
            continue
        flops = per_tok * b * L + shard.n_layers * b * 4.0 * shard.hq * m.head_dim * L * (L + 1) / 2
        rows.append({"tp_degree": shard.tp, "batch": b, "length": L, "latency_us": round(us, 1),
                     "tokens_per_s": round(b * L / us * 1e6, 1), "passes": -(-b * L // width),
                     "tflops": round(flops / us * 1e-6, 2), "frac_of_bf16_mfma_peak": round(flops / us * 1e6 / MFMA_BF16_PEAK, 4)})
    print(json.dumps({"config": args.config, "tp_degree": shard.tp, "n_layers": shard.n_layers, "pass_width": width, "rows": rows}))
    dec.close()


if __name__ == "__main__":
    main()
