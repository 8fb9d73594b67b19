"""Feeds seeded synthetic tensors (pat_inputs) into a Decoder: marshalling only."""
from __future__ import annotations

import numpy as np
import torch

import pat_inputs as pi


def load_synthetic_weights(dec, shard, device="cuda:0"):
    """Generates each layer's shard tensors on the device and hands them to the library,
    one layer at a time (the row-major staging copy is dropped after packing)."""
    for l in range(shard.n_layers):
        w = pi.layer_weights(shard, l, device=device)
        dec.pat_load_layer(l, w)
        torch.cuda.current_stream().synchronize()
        del w
    fw = pi.final_weights(shard, device=device)
    fw["embed"] = pi.embedding_table(shard, device=device)
    dec.pat_load_final(fw)
    torch.cuda.current_stream().synchronize()


def admit_synthetic(dec, shard, req, device="cuda:0", idx=None):
    """Admits requests `idx` of `req` (pat_inputs.rollout_requests) and writes their K/V prefixes."""
    idx = np.arange(len(req["seq_id"])) if idx is None else np.asarray(idx)
    slot0 = dec.pat_get_state()["live"]
    dec.pat_decode_admit(req["seq_id"][idx], req["token"][idx], req["kv_len"][idx], req["target"][idx])
    for j, i in enumerate(idx):
        L = int(req["kv_len"][i])
        if L == 0:
            continue
        for l in range(shard.n_layers):
            k, v = pi.kv_prefix(shard, int(req["seq_id"][i]), l, L, device=device)
            dec.pat_kv_write(slot0 + j, l, k.contiguous(), v.contiguous())
        torch.cuda.current_stream().synchronize()
