"""Micro-benchmark of the weight-streaming projection kernels on the shapes of a configuration.

    python -m paper_2605_23945_amd.kernel_bench [--config 7b_tp1] [--batch 1,16,32,64,256] [--iters 30]
                                                 [--only gateup,down,...,barrier] [--copy-gib 1]

Each projection is run on 6 distinct weight copies in rotation (more than the 256 MB
memory-side cache holds), timed with events on the launch stream.  `--copy-gib` first runs a
plain device-to-device copy of known size: under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its
counters calibrate the unit of the projection kernels' counters.  `--only barrier` times the device-wide barrier
of the fused layer kernel instead (pat_op_barrier_probe) among 32, 64, 128 and 256 resident workgroups.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import torch
    import pat_inputs as pi
    import paper_2605_23945_amd as pat

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="7b_tp1")
    ap.add_argument("--batch", default="1,16,32,64,256")
    ap.add_argument("--iters", type=int, default=30)
    ap.add_argument("--only", default="")
    ap.add_argument("--copy-gib", type=float, default=0.0)
    ap.add_argument("--copies", type=int, default=6, help="distinct weight copies used in rotation (1 = cache-resident if it fits)")
    args = ap.parse_args()
    lib = pat.load_library()
    dev = "cuda:0"
    s = pi.CONFIGS[args.config]["shard"]
    H, d = s.hidden, s.head_dim
    shapes = {"qkv": (s.qkv_rows, H, 0), "o": (H, s.hq * d, 1), "gateup": (2 * s.ffn, H, 2), "down": (H, s.ffn, 1),
              "lm_head": (s.vocab, H, 0)}
    only = [x for x in args.only.split(",") if x]
    stream = torch.cuda.current_stream().cuda_stream
    if args.copy_gib > 0:
        n = int(args.copy_gib * (1 << 30))
        a = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(f"copy  {n} bytes read + {n} bytes written per launch", flush=True)
        del a, b
    if "barrier" in only:
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        for n_wg in (32, 64, 128, 256):
            if n_wg > n_cu:
                continue
            us = [pat.pat_op_barrier_probe(n_wg, iters=500) for _ in range(3)]
            print(f"barrier  workgroups={n_wg:4d}  {min(us):6.2f} us per barrier (best of 3 x 500; others {sorted(us)[1]:.2f}, {max(us):.2f})", flush=True)
        only = [x for x in only if x != "barrier"]
        if not only:
            return
    ncopy = max(1, args.copies)
    for name, (n, k, mode) in shapes.items():
        if only and name not in only:
            continue
        wps = []
        for c in range(ncopy):
            idx = torch.arange(n * k, dtype=torch.int64, device=dev)
            w = pi.normal_bf16(pi.stream_key(77, c, len(name)), idx, 0.02).view(n, k)
            wps.append(pat.pat_op_pack_weight(w[: n // 2], w[n // 2:]) if mode == 2 else pat.pat_op_pack_weight(w))
            del w, idx
        for b in [int(x) for x in args.batch.split(",")]:
            x = torch.randn(b, k, device=dev, generator=torch.Generator(device=dev).manual_seed(b))
            hi, lo = pat.pat_op_pack_act(x)
            y = torch.zeros(b, n, device=dev) if mode != 2 else None
            nb = lib.pat_op_packed_act_bytes(b, n // 2) if mode == 2 else 0
            yh = torch.zeros(max(nb, 16), dtype=torch.uint8, device=dev)
            yl = torch.zeros_like(yh)
            sb = lib.pat_op_gemm_scratch_bytes(n, k, b)
            scratch = torch.empty(max(sb, 256), dtype=torch.uint8, device=dev)

            def run(i):
                rc = lib.pat_op_gemm(wps[i % ncopy].data_ptr(), n, k, hi.data_ptr(), lo.data_ptr(), b,
                                     y.data_ptr() if y is not None else None, n if y is not None else 0,
                                     yh.data_ptr() if mode == 2 else None, yl.data_ptr() if mode == 2 else None, mode,
                                     scratch.data_ptr() if sb > 0 else None, stream)
                assert rc == 0, rc

            for i in range(ncopy):
                run(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(args.iters):
                run(i)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.iters
            plan = (ctypes.c_int32 * 4)()
            lib.pat_op_gemm_plan(n, k, b, plan)
            print(f"{name:8s} N={n:6d} K={k:6d} B={b:4d}  {us:8.1f} us  weights {n * k * 2} B  {n * k * 2 / us / 1e6:6.2f} TB/s  "
                  f"{n * k * 2 / us / 1e6 / 8.0:6.1%} of 8 TB/s  plan(kernel,Kb,Rg,tiles)={list(plan)}", flush=True)


if __name__ == "__main__":
    main()
