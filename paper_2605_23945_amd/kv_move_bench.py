"""Bandwidth of the KV hand-over kernels (gather valid K/V of chosen slots / fill a head slice).

    python -m paper_2605_23945_amd.kv_move_bench [--config 7b_tp1] [--batch 16] [--kv-len 3000] [--heads 0] [--iters 5]

Admits `batch` sequences of `kv-len` cached tokens (page contents are whatever the pool holds: timing
only), gathers all layers of `heads` KV heads (0 = all of the shard's) into one buffer and fills them
back.  Algorithmic bytes = payload read + payload written; HIP events on the launch stream.
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
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--kv-len", type=int, default=3000)
    ap.add_argument("--heads", type=int, default=0)
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    shard = pi.CONFIGS[args.config]["shard"]
    b, L = args.batch, args.kv_len
    nh = args.heads or shard.hkv
    dec = pat.Decoder(pat.make_cfg(shard, b, L + 8, b * L + 64 * b, 64))
    ids = np.arange(b, dtype=np.int32)
    dec.pat_decode_admit(ids, np.zeros(b, np.int32), np.full(b, L, np.int32), np.full(b, 4, np.int32))
    slots = list(range(b))[::-1]                       # not the storage order
    buf, t = dec.pat_kv_extract(slots, n_heads=nh)
    payload = buf.numel() * 2
    res = {}
    for name, fn in (("extract", lambda: dec.pat_kv_extract(slots, n_heads=nh, buf=buf)), ("inject", lambda: dec.pat_kv_inject(slots, buf, n_heads=nh))):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.iters
        res[name] = {"ms": round(ms, 3), "GBps_read_plus_write": round(2 * payload / ms / 1e6, 1), "frac_of_8TBps": round(2 * payload / ms / 1e6 / 8000, 4)}
    # a plain device-to-device copy of the same payload, for scale
    dst = torch.empty_like(buf)
    dst.copy_(buf)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.iters):
        dst.copy_(buf)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.iters
    res["plain_copy"] = {"ms": round(ms, 3), "GBps_read_plus_write": round(2 * payload / ms / 1e6, 1)}
    print(json.dumps({"config": args.config, "batch": b, "kv_len": L, "layers": shard.n_layers, "heads": nh, "tokens": t,
                      "payload_bytes": payload, **res}))
    dec.close()


if __name__ == "__main__":
    main()
