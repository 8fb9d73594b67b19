"""Seeded synthetic inputs for the decode-step path (weights, KV prefixes, token
ids, prompt and response lengths).

This module is the only thing the CPU oracle's tests and the HIP path's callers
share.  It holds no arithmetic of the decode step itself: it only turns
(seed, tensor id, element index) into values, so that any tensor-parallel shard
of any tensor can be produced on its own, on the CPU or on a GPU, with identical
bytes.

Generator: a 32-bit integer hash of the element's flat index in the FULL
(unsharded) tensor, keyed by (seed, tensor id), selects one of 65536 equally
probable normal quantiles  z_k = Phi^-1((k + 0.5) / 65536).  Only integer
arithmetic and a table gather run per element, so CPU and GPU agree bit for bit.
"""
from .generator import (  # noqa: F401
    stream_key,
    hash_u32,
    normal_table_f64,
    normal_bf16,
    uniform_int,
    lognormal_lengths,
)
from .workload import (  # noqa: F401
    ModelShape,
    ShardShape,
    CONFIGS,
    SEED_WEIGHTS,
    SEED_KV,
    SEED_TOKENS,
    shard_of,
    embedding_rows,
    embedding_table,
    layer_weights,
    final_weights,
    kv_prefix,
    prompt_tokens,
    rollout_requests,
)
