"""Shapes and synthetic tensors of the decode workloads.

A `ModelShape` is the full (unsharded) decoder; a `ShardShape` is what one GPU of
a tensor-parallel group of `tp` GPUs holds: its query/KV heads, its slice of the
FFN width and of the vocabulary.  Every shard tensor is an index slice of the
full tensor's value stream, so the shards of one model add up to that model.

Stand-ins: the paper measures on rollouts of trained 8B/14B checkpoints over a
public maths dataset; neither is available here, so weights are N(0, 0.02^2)
rounded to bf16, cached K/V are N(0, 1) rounded to bf16, token ids are uniform
and response lengths are lognormal with the parameters each configuration names.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass

import numpy as np
import torch

from .generator import lognormal_lengths, normal_bf16, stream_key, uniform_int

SEED_WEIGHTS = 0x5EED0001
SEED_KV = 0x5EED0002
SEED_TOKENS = 0x5EED0003

# tensor kinds inside one layer's stream id
_G1, _WQ, _WK, _WV, _WO, _G2, _WG, _WU, _WD, _WLM, _EMB, _GQ, _GK = range(1, 14)


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    qk_norm: bool = False      # per-head RMSNorm of q and k before the rotary embedding (gains gq, gk [head_dim])


@dataclass(frozen=True)
class ShardShape:
    model: ModelShape
    tp: int
    rank: int

    @property
    def n_layers(self): return self.model.n_layers
    @property
    def hidden(self): return self.model.hidden
    @property
    def head_dim(self): return self.model.head_dim
    @property
    def hq(self): return self.model.n_q_heads // self.tp
    @property
    def hkv(self): return max(1, self.model.n_kv_heads // self.tp)
    @property
    def ffn(self): return self.model.ffn // self.tp
    @property
    def vocab(self): return self.model.vocab // self.tp
    @property
    def q_head0(self): return self.rank * self.hq
    @property
    def kv_head0(self):
        m = self.model
        if m.n_kv_heads >= self.tp:
            return self.rank * self.hkv
        return self.rank // (self.tp // m.n_kv_heads)   # replicated KV heads
    @property
    def qkv_rows(self): return (self.hq + 2 * self.hkv) * self.head_dim

    def with_layers(self, n_layers: int) -> "ShardShape":
        return dataclasses.replace(self, model=dataclasses.replace(self.model, n_layers=n_layers))


def shard_of(model: ModelShape, tp: int = 1, rank: int = 0) -> ShardShape:
    assert model.n_q_heads % tp == 0 and model.ffn % tp == 0 and model.vocab % tp == 0
    assert 0 <= rank < tp
    assert model.n_kv_heads % tp == 0 or tp % model.n_kv_heads == 0
    return ShardShape(model, tp, rank)


_TINY = ModelShape(2, 256, 4, 4, 64, 1024, 1024)
_L7B = ModelShape(32, 4096, 32, 32, 128, 11008, 32000)
_L13B = ModelShape(40, 5120, 40, 40, 128, 13824, 32000)
_L70B = ModelShape(80, 8192, 64, 8, 128, 28672, 128256)

# name -> (shard, workload recipe)
CONFIGS = {
    "tiny_tp1": dict(shard=shard_of(_TINY, 1, 0), n_prompts=8, prompt_len=(16, 128),
                     steps=32),
    "7b_tp1": dict(shard=shard_of(_L7B, 1, 0), n_prompts=256, prompt_len=(128, 1024),
                   resp=(6.0, 0.8, 4096)),
    "7b_tp4": dict(shard=shard_of(_L7B, 4, 0), grid_b=(1, 2, 4, 8, 16, 32, 64, 128, 256),
                   grid_l=(512, 2048, 8192)),
    "13b_tp2": dict(shard=shard_of(_L13B, 2, 0), n_prompts=512, prompt_len=(256, 2048),
                    resp=(6.5, 1.0, 8192)),
    "70b_tp8": dict(shard=shard_of(_L70B, 8, 0), n_prompts=1024, prompt_len=(256, 2048),
                    resp=(7.0, 1.0, 16384), grid_b=(1, 2, 4, 8, 16, 32, 64, 128, 256),
                    grid_l=(512, 2048, 8192, 16384)),
}


def _rows(key, r0, r1, ncols, std, mean, device):
    idx = torch.arange(r0 * ncols, r1 * ncols, dtype=torch.int64, device=device)
    return normal_bf16(key, idx, std, mean).view(r1 - r0, ncols)


def _cols(key, nrows, ncols, c0, c1, std, device):
    r = torch.arange(nrows, dtype=torch.int64, device=device)[:, None] * ncols
    c = torch.arange(c0, c1, dtype=torch.int64, device=device)[None, :]
    return normal_bf16(key, (r + c).reshape(-1), std).view(nrows, c1 - c0)


def embedding_table(s: ShardShape, device="cpu", seed=SEED_WEIGHTS) -> torch.Tensor:
    """The full [vocab, hidden] bf16 embedding table (replicated on every shard)."""
    m = s.model
    return _rows(stream_key(seed, 0, _EMB), 0, m.vocab, m.hidden, 0.02, 0.0, device)


def embedding_rows(s: ShardShape, tokens, device="cpu", seed=SEED_WEIGHTS) -> torch.Tensor:
    """Rows `tokens` of the embedding table without building the table."""
    m = s.model
    t = torch.as_tensor(np.asarray(tokens), dtype=torch.int64, device=device)[:, None] * m.hidden
    c = torch.arange(m.hidden, dtype=torch.int64, device=device)[None, :]
    return normal_bf16(stream_key(seed, 0, _EMB), (t + c).reshape(-1), 0.02).view(-1, m.hidden)


def layer_weights(s: ShardShape, layer: int, device="cpu", seed=SEED_WEIGHTS) -> dict:
    """Shard `s`'s tensors of one layer, row-major bf16:

    g1, g2 [H] (and gq, gk [d] if the model normalises q and k per head); wqkv [(hq + 2 hkv) d, H] (q rows, then k rows, then v rows of this
    shard's heads); wo [H, hq d] (this shard's columns); wg, wu [F_s, H];
    wd [H, F_s] (this shard's columns).
    """
    m, d, H = s.model, s.head_dim, s.hidden
    k = lambda kind: stream_key(seed, layer + 1, kind)
    q0, kv0, f0 = s.q_head0 * d, s.kv_head0 * d, s.rank * s.ffn
    wq = _rows(k(_WQ), q0, q0 + s.hq * d, H, 0.02, 0.0, device)
    wk = _rows(k(_WK), kv0, kv0 + s.hkv * d, H, 0.02, 0.0, device)
    wv = _rows(k(_WV), kv0, kv0 + s.hkv * d, H, 0.02, 0.0, device)
    extra = {}
    if m.qk_norm:                      # shared by all heads, hence by all shards
        extra = dict(gq=_rows(k(_GQ), 0, 1, d, 0.02, 1.0, device).view(d), gk=_rows(k(_GK), 0, 1, d, 0.02, 1.0, device).view(d))
    return dict(
        **extra,
        g1=_rows(k(_G1), 0, 1, H, 0.02, 1.0, device).view(H),
        g2=_rows(k(_G2), 0, 1, H, 0.02, 1.0, device).view(H),
        wqkv=torch.cat([wq, wk, wv], 0).contiguous(),
        wo=_cols(k(_WO), H, m.n_q_heads * d, q0, q0 + s.hq * d, 0.02, device).contiguous(),
        wg=_rows(k(_WG), f0, f0 + s.ffn, H, 0.02, 0.0, device),
        wu=_rows(k(_WU), f0, f0 + s.ffn, H, 0.02, 0.0, device),
        wd=_cols(k(_WD), H, m.ffn, f0, f0 + s.ffn, 0.02, device).contiguous(),
    )


def final_weights(s: ShardShape, device="cpu", seed=SEED_WEIGHTS) -> dict:
    """gf [H] and this shard's vocabulary rows wlm [V_s, H]."""
    H = s.hidden
    v0 = s.rank * s.vocab
    return dict(
        gf=_rows(stream_key(seed, 0, _G1), 0, 1, H, 0.02, 1.0, device).view(H),
        wlm=_rows(stream_key(seed, 0, _WLM), v0, v0 + s.vocab, H, 0.02, 0.0, device),
    )


def kv_prefix(s: ShardShape, seq_id: int, layer: int, length: int, device="cpu", seed=SEED_KV):
    """Cached K and V of one sequence in one layer: two bf16 [length, hkv, d] tensors
    ~N(0,1), this shard's KV heads of the full model's stream (K is taken to be
    already position-encoded)."""
    m, d = s.model, s.head_dim
    t = torch.arange(length, dtype=torch.int64, device=device)[:, None] * (m.n_kv_heads * d)
    c = torch.arange(s.kv_head0 * d, (s.kv_head0 + s.hkv) * d, dtype=torch.int64, device=device)[None, :]
    idx = (t + c).reshape(-1)
    kk = normal_bf16(stream_key(seed, seq_id, layer, 0), idx, 1.0).view(length, s.hkv, d)
    vv = normal_bf16(stream_key(seed, seq_id, layer, 1), idx, 1.0).view(length, s.hkv, d)
    return kk, vv


def prompt_tokens(s: ShardShape, seq_id: int, n: int, seed=SEED_TOKENS):
    """The n token ids of one request's prompt (uniform over the vocabulary), for the prefill path."""
    return uniform_int(stream_key(seed, 1000 + int(seq_id)), int(n), 0, s.model.vocab - 1).astype(np.int32)


def rollout_requests(s: ShardShape, n: int, prompt_len, resp=None, steps=None, seed=SEED_TOKENS):
    """n requests: (seq_id, first input token, prompt KV length, response length).

    prompt lengths uniform on [a, b] inclusive; response lengths lognormal(mu,
    sigma) rounded and clamped to [1, cap], or the fixed `steps`.
    """
    tok = uniform_int(stream_key(seed, 1), n, 0, s.model.vocab - 1)
    plen = uniform_int(stream_key(seed, 2), n, prompt_len[0], prompt_len[1])
    if resp is not None:
        tgt = lognormal_lengths(stream_key(seed, 3), n, resp[0], resp[1], resp[2])
    else:
        tgt = np.full(n, int(steps), dtype=np.int64)
    return dict(seq_id=np.arange(n, dtype=np.int32), token=tok.astype(np.int32),
                kv_len=plen.astype(np.int32), target=tgt.astype(np.int32))
