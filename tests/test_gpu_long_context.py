"""Parity at the longest contexts the configurations reach, and the exact-bytes check of the KV append.

Sampled rows at true widths and reduced depth (rows of a batch are independent): 8 192 cached tokens on the
7B TP=4 shard (the last column of configuration 3's grid), 16 300 on the 70B TP=8 shard (configuration 5's
cap), and 256 sequences of about 2 000 tokens on the 70B shard, where the host picks 1024-token attention
chunks.  These reach the rotary table at large positions, page tables of 128 .. 256 pages, and merges of
64 .. 256 chunk partials per row."""
import numpy as np
import pytest
import torch

import pat_inputs as pi
from gpu_util import DEV, check_logits, make_decoder, make_oracle_decoder, oracle_admit
from oracle import bits

pytestmark = pytest.mark.gpu


def _pat():
    import paper_2605_23945_amd as p
    return p


def _run(shard, n, prompt_len, rows, page_tokens=64, steps=1):
    pat = _pat()
    req = pi.rollout_requests(shard, n, prompt_len, steps=steps + 2)
    dec = make_decoder(shard, n, prompt_len[1] + steps + 8, int(req["kv_len"].sum()) + 2 * page_tokens * n + 256, page_tokens)
    pat.admit_synthetic(dec, shard, req, DEV)
    odec = make_oracle_decoder(shard, layer_cache=False)
    oracle_admit(odec, shard, req, rows, steps + 2)
    worst = 0.0
    for _ in range(steps):
        ref_logits, ref_next, _ = odec.step()
        logits = torch.empty(n, shard.vocab, device=DEV)
        nxt = torch.empty(n, dtype=torch.int32, device=DEV)
        dec.pat_decode_step(True, nxt, logits)
        worst = max(worst, check_logits(logits.cpu().numpy()[rows], ref_logits))
        assert np.array_equal(nxt.cpu().numpy()[rows], ref_next)
    dec.close()
    return worst, req


def test_7b_tp4_shard_context_8192():
    shard = pi.shard_of(pi.CONFIGS["7b_tp4"]["shard"].model, 4, 1).with_layers(2)
    worst, req = _run(shard, 3, (8150, 8192), [0, 1, 2], steps=2)
    assert req["kv_len"].max() > 8150
    print(f"7B TP=4, 8192 tokens: worst {worst:.2e} x scale")


def test_7b_tp4_shard_context_8192_live_batch_20():
    """Two batch tiles at the long context (the B <= 32 projection path with 128+ chunks per row)."""
    shard = pi.shard_of(pi.CONFIGS["7b_tp4"]["shard"].model, 4, 0).with_layers(2)
    _run(shard, 20, (7000, 8192), [0, 19])


def test_70b_tp8_shard_context_16300():
    shard = pi.shard_of(pi.CONFIGS["70b_tp8"]["shard"].model, 8, 5).with_layers(2)
    worst, req = _run(shard, 3, (16200, 16370), [0, 1, 2], steps=2)
    assert req["kv_len"].max() > 16200
    print(f"70B TP=8, 16.3k tokens: worst {worst:.2e} x scale")


def test_70b_tp8_shard_256_sequences_of_2000_tokens_take_1024_token_chunks():
    shard = pi.shard_of(pi.CONFIGS["70b_tp8"]["shard"].model, 8, 0).with_layers(2)
    _run(shard, 256, (1900, 2040), [0, 100, 255])


# ---- KV append: the bytes in the page are the bf16 rounding of the path's own fp32 k, v ----------------

def _rot_f32(x0, x1, c, s):
    """The append's rotation as the kernel states it: every product and sum rounded to fp32 on its own."""
    x0, x1, c, s = (np.asarray(a, np.float32) for a in (x0, x1, c, s))
    return (x0 * c).astype(np.float32) - (x1 * s).astype(np.float32), (x0 * s).astype(np.float32) + (x1 * c).astype(np.float32)


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 64), (8, 1, 128), (4, 4, 128)])
def test_kv_append_bytes_are_the_rounding_of_the_projection_output(orc, hq, hkv, d):
    """The fused QKV epilogue writes k (rotated) and v of the new token as bf16.  The same projection run as
    a plain operator gives the path's own fp32 q | k | v; rounding those with the oracle's bf16 conversion
    (k after the rotation at the token's position) must reproduce the appended bytes exactly: no tolerance."""
    pat = _pat()
    H = 256
    m = pi.ModelShape(1, H, hq, hkv, d, 512, 512)
    shard = pi.shard_of(m, 1, 0)
    lens = np.array([0, 1, 63, 64, 200, 777, 1030], np.int32)
    n = len(lens)
    req = pi.rollout_requests(shard, n, (1, 2), steps=3)
    req["kv_len"] = lens
    dec = make_decoder(shard, n, 1100, int(lens.sum()) + 64 * n + 256)
    pat.admit_synthetic(dec, shard, req, DEV)
    dec.pat_decode_step(True)
    # the path's own fp32 k, v: the same two operators the step runs (embedding rows with their sums of squares,
    # then the projection with the RMSNorm folded in), without the rotary / append epilogue
    w = pi.layer_weights(shard, 0, device=DEV)
    table = pi.embedding_table(shard, device=DEV)
    x, stats, xg_hi, xg_lo = pat.pat_op_embed_stats(table, torch.as_tensor(req["token"], dtype=torch.int32, device=DEV), w["g1"])
    y = pat.pat_op_gemm_norm(pat.pat_op_pack_weight(w["wqkv"]), shard.qkv_rows, H, xg_hi, xg_lo, stats, m.rms_eps, n,
                             fused=dec.pat_decode_uses_fused_kernel())
    y = y.cpu().numpy()
    half = d // 2
    inv = np.power(np.float64(m.rope_base), -2.0 * np.arange(half) / d)
    for i in range(n):
        L = int(lens[i])
        kc, vc = dec.pat_kv_read(i, 0, L + 1)
        k_got, v_got = bits(kc)[L], bits(vc)[L]                       # [hkv, d] of the appended position
        ang = np.float64(L) * inv
        c, s = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
        for h in range(hkv):
            kf = y[i, (hq + h) * d:(hq + h + 1) * d]
            vf = y[i, (hq + hkv + h) * d:(hq + hkv + h + 1) * d]
            r0, r1 = _rot_f32(kf[:half], kf[half:], c, s)
            k_want = np.array([orc.real_to_bf16(float(t)) for t in np.concatenate([r0, r1])], np.uint16)
            v_want = np.array([orc.real_to_bf16(float(t)) for t in vf], np.uint16)
            assert np.array_equal(v_got[h], v_want), (i, h, "v")
            assert np.array_equal(k_got[h], k_want), (i, h, "k")
    dec.close()
