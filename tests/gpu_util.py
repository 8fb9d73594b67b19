"""Helpers of the GPU parity tests: one set of seeded inputs feeds both the HIP
library (through its C ABI) and the CPU oracle.  No value flows from one side
to the other."""
from __future__ import annotations

import numpy as np
import torch

import pat_inputs as pi
from oracle import Oracle, OracleDecoder, bits

DEV = "cuda:0"

# Logit tolerance of the benchmark spec: max-abs <= 2e-2 x the logit scale (std of the
# oracle's logits of that row).  The arithmetic of this implementation (split-bf16 operands,
# fp32 accumulation) is good to about 1e-4 of the scale; what is left is the KV append: a k or v
# element within that distance of a bf16 rounding boundary rounds the other way than in the
# float64 oracle (one bf16 step = 2^-8 of the element), and with only a few cached tokens a
# single such element moves the logits by up to ~1e-3 of the scale.  DESIGN_TOL bounds that.
TOL = 2e-2
DESIGN_TOL = 5e-3
KV_ABS_TOL = 5e-4


def widen(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def make_decoder(shard, max_batch, max_seq_len, budget, page_tokens=64, eos=-1):
    import paper_2605_23945_amd as pat
    cfg = pat.make_cfg(shard, max_batch, max_seq_len, budget, page_tokens, eos)
    dec = pat.Decoder(cfg, DEV)
    pat.load_synthetic_weights(dec, shard, DEV)
    return dec


def make_oracle_decoder(shard, eos=-1, precision="f64", layer_cache=True):
    m = shard.model
    cache = {}

    def layer_w(l):
        if l not in cache:
            if not layer_cache:
                cache.clear()
            cache[l] = {k: bits(v) for k, v in pi.layer_weights(shard, l, device=_gen_device()).items()}
        return cache[l]

    fw = {k: bits(v) for k, v in pi.final_weights(shard, device=_gen_device()).items()}
    emb = lambda t: bits(pi.embedding_rows(shard, [t]))[0]
    return OracleDecoder(Oracle(precision), (m.n_layers, m.hidden, shard.hq, shard.hkv, m.head_dim, shard.ffn,
                                             m.rms_eps, m.rope_base), layer_w, fw, emb,
                         vocab0=shard.rank * shard.vocab, eos=eos)


def _gen_device():
    # big tensors are generated on the GPU (same integer arithmetic, same bytes) and copied to the host
    return DEV if torch.cuda.is_available() else "cpu"


def oracle_admit(odec, shard, req, idx, cap_extra):
    for i in idx:
        L = int(req["kv_len"][i])
        kv = [pi.kv_prefix(shard, int(req["seq_id"][i]), l, L) for l in range(shard.n_layers)]
        odec.admit(req["seq_id"][i], req["token"][i], L, req["target"][i],
                   [bits(a) for a, _ in kv], [bits(b) for _, b in kv], cap_extra)


def check_logits(got: np.ndarray, ref: np.ndarray, tol=TOL, design_tol=DESIGN_TOL):
    """Row-wise max-abs error relative to the row's logit scale. Returns the worst ratio."""
    worst = 0.0
    for i in range(ref.shape[0]):
        s = float(ref[i].std())
        e = float(np.max(np.abs(got[i].astype(np.float64) - ref[i])))
        worst = max(worst, e / s)
    assert worst <= tol, f"logit error {worst:.3e} x scale exceeds the stated tolerance {tol}"
    assert worst <= design_tol, f"logit error {worst:.3e} x scale exceeds what split-bf16/fp32 arithmetic should give"
    return worst


def bf16_close(a_bits: np.ndarray, b_bits: np.ndarray, abs_tol=KV_ABS_TOL):
    """(fraction bit-identical, all within one bf16 step).

    The fp32 k, v that get rounded already differ from the oracle's by the path's accumulated
    arithmetic error (KV_ABS_TOL, relative to the tensor's scale), which matters
    for elements that cancel to nearly zero; so the allowance is one bf16 step of the value
    plus KV_ABS_TOL of the tensor's rms."""
    same = a_bits == b_bits
    a, b = widen(a_bits), widen(b_bits)
    step = np.maximum(np.abs(a), np.abs(b)) * 2.0 ** -7 + abs_tol * float(np.sqrt(np.mean(b * b)))
    return float(same.mean()), bool(np.all(np.abs(a - b) <= step))
