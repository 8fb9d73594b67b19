"""KV migration, the local half (gather valid K/V of chosen slots; fill a head slice of admitted slots):
bit-exact against the oracle's element-by-element gather, then a full hand-over between shard shapes."""
import numpy as np
import pytest
import torch

import pat_inputs as pi
from gpu_util import DEV, check_logits, make_decoder, make_oracle_decoder, oracle_admit
from oracle import bits, kv_extract

pytestmark = pytest.mark.gpu


def _pat():
    import paper_2605_23945_amd as p
    p.load_library()
    return p


def _requests(shard, lens, steps=4):
    req = pi.rollout_requests(shard, len(lens), (1, 2), steps=steps)
    req["kv_len"] = np.asarray(lens, np.int32)
    return req


def test_extract_is_bit_exact_for_any_selection_order_and_slice():
    shard = pi.CONFIGS["tiny_tp1"]["shard"]                       # 2 layers, 4 KV heads x 64
    pat = _pat()
    lens = [37, 0, 16, 129, 1, 64, 95]                            # page size 16: empty, exact pages, ragged tails
    req = _requests(shard, lens)
    dec = make_decoder(shard, 8, 256, 1024, page_tokens=16)
    pat.admit_synthetic(dec, shard, req, DEV)
    odec = make_oracle_decoder(shard)
    oracle_admit(odec, shard, req, range(len(lens)), 4)
    for slots, l0, nl, h0, nh in [([0, 1, 2, 3, 4, 5, 6], 0, 2, 0, 4), ([3], 1, 1, 2, 1), ([6, 0, 3], 0, 2, 1, 2),
                                  ([1], 0, 2, 0, 4), ([5, 4, 2], 0, 1, 3, 1)]:
        buf, t = dec.pat_kv_extract(slots, l0, nl, h0, nh)
        ref = kv_extract(odec, slots, l0, nl, h0, nh)
        assert t == ref.shape[3] == sum(lens[s] for s in slots)
        assert np.array_equal(bits(buf.cpu()), ref), (slots, l0, nl, h0, nh)
    # the pool is untouched: a second full extract gives the same bytes
    a, _ = dec.pat_kv_extract(list(range(7)))
    b, _ = dec.pat_kv_extract(list(range(7)))
    assert torch.equal(a, b)
    dec.close()


def test_error_paths():
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    pat = _pat()
    req = _requests(shard, [20, 30])
    dec = make_decoder(shard, 4, 128, 512, page_tokens=16)
    pat.admit_synthetic(dec, shard, req, DEV)
    buf, t = dec.pat_kv_extract([0, 1])
    for bad in (lambda: dec.pat_kv_extract([0, 0]), lambda: dec.pat_kv_extract([2]), lambda: dec.pat_kv_extract([0], head0=3, n_heads=2),
                lambda: dec.pat_kv_extract([0], layer0=1, n_layers=2), lambda: dec.pat_kv_extract([0, 1], buf=buf[:, :, :, :10].contiguous()),
                lambda: dec.pat_kv_inject([0], buf),                                    # 50 tokens for a slot of 20
                lambda: dec.pat_kv_inject([0, 1], buf, pool_head0=2, n_heads=3)):
        with pytest.raises(pat.PatError) as e:
            bad()
        assert e.value.code == pat.binding.PAT_EINVAL
    again, _ = dec.pat_kv_extract([0, 1])
    assert torch.equal(buf, again)                                 # nothing was changed by the rejected calls
    dec.close()


def test_hand_over_tp1_to_a_tp2_rank_and_decode_on():
    """Sequences held by a TP=1 engine move to rank 1 of a TP=2 layout: gather heads 2..3, admit on the
    target, fill its two heads, then decode there; the oracle of the target shard starts from the
    same slice."""
    model = pi.CONFIGS["tiny_tp1"]["shard"].model
    src_shard = pi.shard_of(model, 1, 0)
    dst_shard = pi.shard_of(model, 2, 1)
    pat = _pat()
    lens = [70, 33, 48]
    req = _requests(src_shard, lens, steps=3)
    src = make_decoder(src_shard, 4, 160, 512, page_tokens=16)
    pat.admit_synthetic(src, src_shard, req, DEV)
    osrc = make_oracle_decoder(src_shard)
    oracle_admit(osrc, src_shard, req, range(3), 4)
    moved = [2, 0]                                                  # the survivors, in their new order
    buf, t = src.pat_kv_extract(moved, head0=dst_shard.kv_head0, n_heads=dst_shard.hkv)
    dst = make_decoder(dst_shard, 4, 160, 512, page_tokens=16)
    sub = {k: v[moved] for k, v in req.items()}
    dst.pat_decode_admit(sub["seq_id"], sub["token"], sub["kv_len"], sub["target"])
    dst.pat_kv_inject([0, 1], buf)
    odst = make_oracle_decoder(dst_shard)
    for j, s in enumerate(moved):
        ks = [osrc.kc[s][l][:lens[s], dst_shard.kv_head0:dst_shard.kv_head0 + dst_shard.hkv] for l in range(model.n_layers)]
        vs = [osrc.vc[s][l][:lens[s], dst_shard.kv_head0:dst_shard.kv_head0 + dst_shard.hkv] for l in range(model.n_layers)]
        odst.admit(sub["seq_id"][j], sub["token"][j], lens[s], sub["target"][j], ks, vs, 4)
        for l in range(model.n_layers):
            k, v = dst.pat_kv_read(j, l, lens[s])
            assert np.array_equal(bits(k.cpu()), ks[l]) and np.array_equal(bits(v.cpu()), vs[l])
    for _ in range(2):
        logits = torch.empty(2, dst_shard.vocab, device=DEV)
        nxt = torch.empty(2, dtype=torch.int32, device=DEV)
        dst.pat_decode_step(report=True, next_tok=nxt, logits=logits)
        ref_logits, ref_next, _ = odst.step()
        check_logits(logits.cpu().numpy(), ref_logits)
        assert np.array_equal(nxt.cpu().numpy(), ref_next)
    src.close(); dst.close()


def test_gather_from_two_tp2_ranks_into_tp1():
    """TP decrease: the buffers of the two source ranks, concatenated along the head axis (what an
    all-gather returns), fill all four heads of a TP=1 engine."""
    model = pi.CONFIGS["tiny_tp1"]["shard"].model
    full = pi.shard_of(model, 1, 0)
    pat = _pat()
    lens = [21, 64, 5]
    parts = []
    for rank in (0, 1):
        sh = pi.shard_of(model, 2, rank)
        req = _requests(sh, lens)
        d = make_decoder(sh, 4, 128, 512, page_tokens=16)
        pat.admit_synthetic(d, sh, req, DEV)
        parts.append(d.pat_kv_extract([0, 1, 2])[0])
        d.close()
    gathered = torch.cat(parts, dim=2).contiguous()                 # [layers, 2, 4 heads, T, d]
    req = _requests(full, lens)
    dst = make_decoder(full, 4, 128, 512, page_tokens=16)
    dst.pat_decode_admit(req["seq_id"], req["token"], req["kv_len"], req["target"])
    dst.pat_kv_inject([0, 1, 2], gathered)
    oref = make_oracle_decoder(full)
    oracle_admit(oref, full, req, range(3), 2)
    got, _ = dst.pat_kv_extract([0, 1, 2])
    assert np.array_equal(bits(got.cpu()), kv_extract(oref, [0, 1, 2], 0, model.n_layers, 0, 4))
    dst.close()
