"""Step-level parity of the HIP decode path (through the C ABI) against the CPU oracle:
logits within tolerance, tokens / integer state / compaction bit-exact, appended K/V
within one bf16 step, allocator invariants, error paths."""
import dataclasses

import numpy as np
import pytest
import torch

import pat_inputs as pi
from gpu_util import (DEV, bf16_close, check_logits, make_decoder, make_oracle_decoder, oracle_admit)
from oracle import bits

pytestmark = pytest.mark.gpu


def _pat():
    import paper_2605_23945_amd as p
    return p


def _gpu_step(dec, B, vs):
    logits = torch.empty(B, vs, device=DEV)
    nxt = torch.empty(B, dtype=torch.int32, device=DEV)
    rep = dec.pat_decode_step(True, nxt, logits)
    return logits.cpu().numpy(), nxt.cpu().numpy(), rep


def _check_pages(dec, P):
    st = dec.pat_get_state()
    pt, free = dec.pat_get_pages()
    used = []
    for i in range(st["live"]):
        used += pt[i, : -(-int(st["kv_len"][i]) // P)].tolist()
    assert len(used) == len(set(used)), "a page is owned twice"
    assert not (set(used) & set(free.tolist())), "a page is both owned and free"
    assert len(set(free.tolist())) == len(free)
    assert len(used) + len(free) == dec.req.n_pages
    return st


def _rollout_parity(shard, n_seq, prompt_len, targets, page_tokens=64, max_steps=10**9, check_kv=True):
    """Free-running greedy rollout on both sides with compaction whenever a sequence finishes."""
    pat = _pat()
    req = pi.rollout_requests(shard, n_seq, prompt_len, steps=1)
    req["target"] = np.asarray(targets, np.int32)
    cap = int(req["target"].max()) + 1
    dec = make_decoder(shard, max(n_seq, 1), int(req["kv_len"].max()) + cap + 1,
                       int((req["kv_len"] + req["target"]).sum()) + 64 * n_seq, page_tokens)
    pat.admit_synthetic(dec, shard, req, DEV)
    odec = make_oracle_decoder(shard)
    oracle_admit(odec, shard, req, range(n_seq), cap)
    worst, step = 0.0, 0
    while len(odec.tok) and step < max_steps:
        B = len(odec.tok)
        ref_logits, ref_next, ref_nf = odec.step()
        got_logits, got_next, rep = _gpu_step(dec, B, shard.vocab)
        worst = max(worst, check_logits(got_logits, ref_logits))
        assert np.array_equal(got_next, ref_next), f"step {step}: tokens differ"
        assert rep.live_batch == B and rep.n_finished == ref_nf and rep.sum_context == int(odec.kv_len.sum())
        st = dec.pat_get_state()
        for k_gpu, k_orc in (("seq_id", "seq_id"), ("token", "tok"), ("kv_len", "kv_len"), ("gen", "gen"),
                             ("target", "target"), ("fin", "fin")):
            assert np.array_equal(st[k_gpu], getattr(odec, k_orc)), k_gpu
        if ref_nf:
            before = {}
            for j in range(B):
                if not odec.fin[j]:
                    before[int(odec.seq_id[j])] = [tuple(t.cpu() for t in dec.pat_kv_read(j, l, int(odec.kv_len[j])))
                                                   for l in range(shard.n_layers)]
            nb = odec.compact()
            assert dec.pat_kv_compact() == nb
            st = _check_pages(dec, page_tokens)
            assert st["live"] == nb
            for k_gpu, k_orc in (("seq_id", "seq_id"), ("token", "tok"), ("kv_len", "kv_len"), ("gen", "gen"),
                                 ("target", "target")):
                assert np.array_equal(st[k_gpu], getattr(odec, k_orc)), k_gpu
            for j in range(nb):        # the survivors' logical K/V is byte-identical after the move
                for l in range(shard.n_layers):
                    k, v = dec.pat_kv_read(j, l, int(odec.kv_len[j]))
                    kb, vb = before[int(odec.seq_id[j])][l]
                    assert torch.equal(k.cpu(), kb) and torch.equal(v.cpu(), vb)
        step += 1
    if check_kv and len(odec.tok):
        for j in range(len(odec.tok)):
            L = int(odec.kv_len[j])
            for l in range(shard.n_layers):
                k, v = dec.pat_kv_read(j, l, L)
                L0 = L - int(odec.gen[j])
                assert np.array_equal(bits(k)[:L0], odec.kc[j][l][:L0])          # the prompt's K/V are untouched
                for got, ref in ((bits(k)[L0:], odec.kc[j][l][L0:L]), (bits(v)[L0:], odec.vc[j][l][L0:L])):
                    frac, close = bf16_close(got, ref)
                    assert close and frac > 0.98, (frac, close)
    dec.close()
    return worst, step


def test_tiny_config_32_greedy_steps():
    """Configuration 1: 2 layers, hidden 256, 4 heads x 64, batch 8, KV lengths U[16,128], 32 steps."""
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    worst, steps = _rollout_parity(shard, 8, (16, 128), [33] * 8, max_steps=32)
    assert steps == 32
    print(f"tiny: worst logit error {worst:.2e} x scale")


def test_tiny_rollout_with_compaction_until_empty():
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    targets = [3, 1, 7, 3, 12, 1, 5, 9, 2, 12, 4]
    worst, steps = _rollout_parity(shard, len(targets), (1, 150), targets, page_tokens=16)
    assert steps == 12


def test_no_prompt_and_page_boundaries():
    """kv_len = 0 (nothing cached) and lengths that sit exactly on page boundaries."""
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    pat = _pat()
    req = pi.rollout_requests(shard, 5, (1, 2), steps=20)
    req["kv_len"] = np.array([0, 15, 16, 17, 32], np.int32)
    dec = make_decoder(shard, 5, 64, 400, 16)
    pat.admit_synthetic(dec, shard, req, DEV)
    odec = make_oracle_decoder(shard)
    oracle_admit(odec, shard, req, range(5), 21)
    for _ in range(20):
        ref_logits, ref_next, _ = odec.step()
        got_logits, got_next, _ = _gpu_step(dec, 5, shard.vocab)
        check_logits(got_logits, ref_logits)
        assert np.array_equal(got_next, ref_next)
    _check_pages(dec, 16)
    dec.close()


@pytest.mark.parametrize("tp,rank", [(2, 1), (4, 3)])
def test_tp_shard_of_tiny_model(tp, rank):
    """A TP shard is the shard's shapes; its vocabulary slice reports global token ids."""
    m = pi.CONFIGS["tiny_tp1"]["shard"].model
    shard = pi.shard_of(m, tp, rank)
    worst, _ = _rollout_parity(shard, 3, (10, 90), [4, 2, 4])


@pytest.mark.parametrize("hq,hkv,d", [(8, 1, 128), (8, 2, 64), (4, 2, 128)])
def test_grouped_query_shapes(hq, hkv, d):
    m = pi.ModelShape(2, 256, hq, hkv, d, 512, 512)
    _rollout_parity(pi.shard_of(m, 1, 0), 4, (30, 300), [3, 3, 2, 3])


@pytest.mark.parametrize("page_tokens", [64, 16])
def test_grouped_query_many_long_sequences_use_long_chunks(page_tokens):
    """One KV head, 8 query heads, 72 sequences of about 3000 cached tokens: more 256-token chunks than
    the chip holds at once, so the host picks 512-token chunks (8 rounds per item, 8 or 32 pages each)."""
    m = pi.ModelShape(1, 256, 8, 1, 128, 512, 512)
    _sampled_rows_parity(pi.shard_of(m, 1, 0), 72, (2800, 3300), [0, 17, 71], steps=2, page_tokens=page_tokens)


def test_long_context_many_chunks_and_ragged_batch():
    """Lengths spanning several attention chunks and pages with a ragged tail; batch 19 = two batch tiles."""
    m = pi.ModelShape(1, 256, 4, 2, 64, 512, 512)
    shard = pi.shard_of(m, 1, 0)
    n = 19
    req = pi.rollout_requests(shard, n, (1, 1500), steps=2)
    _rollout_parity(shard, n, (1, 1500), [2] * n, check_kv=False)


def test_determinism_bitwise():
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    pat = _pat()
    outs = []
    for _ in range(2):
        req = pi.rollout_requests(shard, 6, (16, 400), steps=3)
        dec = make_decoder(shard, 6, 512, 4096)
        pat.admit_synthetic(dec, shard, req, DEV)
        acc = [_gpu_step(dec, 6, shard.vocab)[0] for _ in range(3)]
        outs.append(np.stack(acc))
        dec.close()
    assert np.array_equal(outs[0], outs[1])


def test_eos_token_finishes_a_sequence():
    """With eos enabled the finish flag follows the token the device chose."""
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    pat = _pat()
    req = pi.rollout_requests(shard, 3, (8, 40), steps=6)
    odec = make_oracle_decoder(shard)
    oracle_admit(odec, shard, req, range(3), 8)
    _, first, _ = odec.step()
    eos = int(first[1])                                  # the token sequence 1 produces first
    odec = make_oracle_decoder(shard, eos=eos)
    oracle_admit(odec, shard, req, range(3), 8)
    dec = make_decoder(shard, 3, 64, 512, 16, eos=eos)
    pat.admit_synthetic(dec, shard, req, DEV)
    _, ref_next, nf = odec.step()
    _, got_next, rep = _gpu_step(dec, 3, shard.vocab)
    assert np.array_equal(got_next, ref_next) and rep.n_finished == nf >= 1
    assert np.array_equal(dec.pat_get_state()["fin"], odec.fin)
    assert dec.pat_kv_compact() == odec.compact()
    assert np.array_equal(dec.pat_get_state()["seq_id"], odec.seq_id)
    dec.close()


def test_error_paths_leave_state_untouched():
    pat = _pat()
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    bad = pat.make_cfg(shard, 4, 64, 256, page_tokens=48)
    with pytest.raises(pat.PatError):
        pat.Decoder(bad, DEV)
    bad = pat.make_cfg(pi.ShardShape(shard.model, 3, 0), 4, 64, 256)          # 4 heads not divisible by 3
    with pytest.raises(pat.PatError):
        pat.Decoder(bad, DEV)
    dec = make_decoder(shard, 4, 64, 64, 16)                                  # pool: 4 + 4 pages of 16 tokens
    with pytest.raises(pat.PatError) as e:
        dec.pat_decode_step()
    assert e.value.code == pat.binding.PAT_ESTATE                              # empty batch
    req = pi.rollout_requests(shard, 6, (10, 20), steps=2)
    with pytest.raises(pat.PatError) as e:
        dec.pat_decode_admit(req["seq_id"], req["token"], req["kv_len"], req["target"])
    assert e.value.code == pat.binding.PAT_ENOMEM                              # 6 > max_batch
    big = dict(req); big["kv_len"] = np.full(6, 40, np.int32)
    with pytest.raises(pat.PatError) as e:
        dec.pat_decode_admit(big["seq_id"][:4], big["token"][:4], big["kv_len"][:4], big["target"][:4])
    assert e.value.code == pat.binding.PAT_ENOMEM                              # 12 pages > 8
    with pytest.raises(pat.PatError) as e:
        dec.pat_decode_admit(req["seq_id"][:1], req["token"][:1], np.array([60], np.int32), np.array([10], np.int32))
    assert e.value.code == pat.binding.PAT_EINVAL                              # 70 > max_seq_len
    assert dec.pat_get_state()["live"] == 0 and len(dec.pat_get_pages()[1]) == dec.req.n_pages
    idx = [0, 1]
    pat.admit_synthetic(dec, shard, req, DEV, idx=idx)
    dec.pat_decode_step(); dec.pat_decode_step()                              # both reach their target of 2
    with pytest.raises(pat.PatError) as e:
        dec.pat_decode_step()
    assert e.value.code == pat.binding.PAT_ESTATE                              # finished slots present
    assert dec.pat_kv_compact() == 0
    assert len(dec.pat_get_pages()[1]) == dec.req.n_pages                      # every page came back
    dec.close()


def test_page_exhaustion_is_reported_before_the_step():
    pat = _pat()
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    dec = make_decoder(shard, 2, 256, 32, 16)                                  # 2 + 2 pages
    req = pi.rollout_requests(shard, 2, (16, 16), steps=100)
    pat.admit_synthetic(dec, shard, req, DEV)                                  # one page each, both full
    dec.pat_decode_step()                                                      # takes the two spare pages
    for _ in range(15):
        dec.pat_decode_step()
    with pytest.raises(pat.PatError) as e:
        dec.pat_decode_step()                                                  # would need two more pages
    assert e.value.code == pat.binding.PAT_ENOMEM
    assert np.array_equal(dec.pat_get_state()["kv_len"], [32, 32])
    dec.close()


def test_7b_shape_two_layers_sampled_rows():
    """True 7B widths (hidden 4096, 32 heads x 128, FFN 11008, vocab 32000) at reduced depth;
    batch 40 (three batch tiles, ragged), oracle on sampled rows (rows are independent)."""
    shard = pi.CONFIGS["7b_tp1"]["shard"].with_layers(2)
    pat = _pat()
    n = 40
    req = pi.rollout_requests(shard, n, (128, 1024), steps=4)
    dec = make_decoder(shard, n, 1100, int(req["kv_len"].sum()) + 64 * n + 256)
    pat.admit_synthetic(dec, shard, req, DEV)
    rows = [0, 15, 16, 39, int(np.argmax(req["kv_len"])), int(np.argmin(req["kv_len"]))]
    odec = make_oracle_decoder(shard)
    oracle_admit(odec, shard, req, rows, 4)
    for step in range(2):
        ref_logits, ref_next, _ = odec.step()
        got_logits, got_next, _ = _gpu_step(dec, n, shard.vocab)
        w = check_logits(got_logits[rows], ref_logits)
        assert np.array_equal(got_next[rows], ref_next)
        print(f"7b x2 layers step {step}: worst {w:.2e} x scale")
    dec.close()


def test_70b_gqa_tp8_shape_two_layers_sampled_rows():
    """70B-style TP=8 shard widths: hidden 8192, 8 query heads sharing 1 KV head, FFN slice 3584,
    vocabulary slice 16032 of rank 3 (global ids offset)."""
    shard = pi.shard_of(pi.CONFIGS["70b_tp8"]["shard"].model, 8, 3).with_layers(2)
    pat = _pat()
    n = 5
    req = pi.rollout_requests(shard, n, (256, 2048), steps=3)
    dec = make_decoder(shard, n, 2100, int(req["kv_len"].sum()) + 64 * n + 256)
    pat.admit_synthetic(dec, shard, req, DEV)
    rows = [0, 4]
    odec = make_oracle_decoder(shard)
    oracle_admit(odec, shard, req, rows, 3)
    ref_logits, ref_next, _ = odec.step()
    got_logits, got_next, _ = _gpu_step(dec, n, shard.vocab)
    check_logits(got_logits[rows], ref_logits)
    assert np.array_equal(got_next[rows], ref_next)
    assert np.all(got_next >= 3 * shard.vocab) and np.all(got_next < 4 * shard.vocab)
    dec.close()


def _sampled_rows_parity(shard, n, prompt_len, rows, steps=1, max_seq=None, page_tokens=64):
    pat = _pat()
    req = pi.rollout_requests(shard, n, prompt_len, steps=steps + 2)
    dec = make_decoder(shard, n, (max_seq or prompt_len[1]) + steps + 8, int(req["kv_len"].sum()) + 2 * page_tokens * n + 256, page_tokens)
    pat.admit_synthetic(dec, shard, req, DEV)
    odec = make_oracle_decoder(shard, layer_cache=False)
    oracle_admit(odec, shard, req, rows, steps + 2)
    worst = 0.0
    for _ in range(steps):
        ref_logits, ref_next, _ = odec.step()
        got_logits, got_next, _ = _gpu_step(dec, n, shard.vocab)
        worst = max(worst, check_logits(got_logits[rows], ref_logits))
        assert np.array_equal(got_next[rows], ref_next)
    dec.close()
    return worst


def test_7b_tp4_shard_shape_two_layers_sampled_rows():
    """Configuration 3's shard: 8 heads x 128, FFN slice 2752, vocabulary slice 8000 (rank 2 of 4)."""
    shard = pi.shard_of(pi.CONFIGS["7b_tp4"]["shard"].model, 4, 2).with_layers(2)
    _sampled_rows_parity(shard, 70, (100, 600), [0, 31, 32, 69], steps=2)     # 70 rows: five batch tiles, two batch groups


def test_7b_shape_two_layers_batch_200_full_batch_projections():
    """Live batch 200 (13 batch tiles, the last one ragged): the projections that hold the whole batch."""
    shard = pi.CONFIGS["7b_tp1"]["shard"].with_layers(2)
    _sampled_rows_parity(shard, 200, (64, 300), [0, 63, 64, 127, 128, 191, 192, 199], steps=2)


def test_live_batch_300_runs_as_two_projection_groups():
    """More than 256 live sequences: the projections run as groups of 256 rows (256 + 44 here), every
    other kernel over all rows at once; rows on both sides of the group boundary are checked."""
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    _sampled_rows_parity(shard, 300, (10, 120), [0, 255, 256, 257, 299], steps=2, page_tokens=16)


def test_13b_tp2_shard_batch_130_full_batch_projections():
    """Live batch 130 (nine batch tiles -> the 12-tile shape) on the hidden-5120 shard."""
    shard = pi.CONFIGS["13b_tp2"]["shard"].with_layers(2)
    _sampled_rows_parity(shard, 130, (64, 200), [0, 64, 128, 129], steps=1)


def test_13b_tp2_shard_shape_two_layers_sampled_rows():
    """Configuration 4's shard: hidden 5120, 20 of 40 heads, FFN slice 6912, vocabulary slice 16000."""
    shard = pi.CONFIGS["13b_tp2"]["shard"].with_layers(2)
    _sampled_rows_parity(shard, 20, (256, 2048), [0, 15, 16, 19])


def test_7b_full_depth_sampled_rows_in_bench_configuration():
    """Configuration 2 at full depth (32 layers) in the launch shapes the benchmark times (live batch
    <= 16 path and the 33..256 path): oracle on sampled rows, one step."""
    shard = pi.CONFIGS["7b_tp1"]["shard"]
    pat = _pat()
    n = 48
    req = pi.rollout_requests(shard, n, (128, 1024), steps=3)
    dec = make_decoder(shard, n, 1100, int(req["kv_len"].sum()) + 64 * n + 256)
    pat.admit_synthetic(dec, shard, req, DEV)
    rows = [0, 47]
    odec = make_oracle_decoder(shard, layer_cache=False)
    oracle_admit(odec, shard, req, rows, 3)
    ref_logits, ref_next, _ = odec.step()
    got_logits, got_next, _ = _gpu_step(dec, n, shard.vocab)              # 48 rows: the batched (LDS-staged) projections
    w1 = check_logits(got_logits[rows], ref_logits)
    assert np.array_equal(got_next[rows], ref_next)
    # the same two sequences alone in a fresh batch: the small-batch streaming projections
    dec.pat_decode_reset()
    sub = {k: v[rows] for k, v in req.items()}
    pat.admit_synthetic(dec, shard, sub, DEV)
    odec2 = make_oracle_decoder(shard, layer_cache=False)
    oracle_admit(odec2, shard, req, rows, 3)
    ref_logits2, ref_next2, _ = odec2.step()
    got_logits2, got_next2, _ = _gpu_step(dec, 2, shard.vocab)
    w2 = check_logits(got_logits2, ref_logits2)
    assert np.array_equal(got_next2, ref_next2)
    assert np.array_equal(ref_next, ref_next2)                            # rows do not depend on their batch
    print(f"7B full depth: worst {max(w1, w2):.2e} x scale")
    dec.close()


@pytest.mark.parametrize("config,n,rows", [("70b_tp8", 40, [0, 39]), ("13b_tp2", 20, [3, 19])])
def test_full_depth_shards_sampled_rows(config, n, rows):
    """The 70B TP=8 shard (80 layers, 8 query heads on 1 KV head: the matrix-score attention kernel) and
    the 13B TP=2 shard (40 layers) at full depth: oracle on two sampled rows, one step; the error after
    80 layers must still meet the logit bar."""
    shard = pi.CONFIGS[config]["shard"]
    worst = _sampled_rows_parity(shard, n, (128, 700), rows, steps=1)
    print(f"{config} full depth: worst {worst:.2e} x scale")


def test_profile_grid_protocol():
    """Offline-profiler sweep: B*L <= T_cap pruning, row order, mean of the timed steps, byte model."""
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    pat = _pat()
    dec = make_decoder(shard, 32, 1024 + 80, 1 << 14)
    Bs, Ls = [1, 4, 32], [16, 256, 1024]
    rows = dec.pat_profile_grid(Bs, Ls, t_cap=1 << 13, steps=12, warmup=2, reps=2, seed=7)
    assert len(rows) == 9
    for i, r in enumerate(rows):
        b, l = Bs[i // 3], Ls[i % 3]
        assert (r["batch"], r["kv_len"], r["tp_degree"]) == (b, l, 1)
        if b * l > (1 << 13):
            assert r["skipped"] == 1 and r["mean_us"] == 0.0
        else:
            assert r["skipped"] == 0 and r["mean_us"] > 0 and r["min_us"] <= r["mean_us"]
            assert r["sum_context"] == b * (l + 2 + 6)                       # context tokens at the middle of the timed window
            assert abs(r["tokens_per_s"] - b / (r["mean_us"] * 1e-6)) < 1e-6 * r["tokens_per_s"]
            m = shard.model
            wbytes = m.n_layers * 2 * (m.hidden * shard.qkv_rows + shard.hq * m.head_dim * m.hidden + 3 * m.hidden * shard.ffn) \
                + 2 * shard.vocab * m.hidden
            kv = m.n_layers * 2 * shard.hkv * m.head_dim * 2 * (b * (l + 2 + 6 + 1) + b)
            assert r["algo_bytes"] == wbytes + kv
    assert [r["skipped"] for r in rows] == [0, 0, 0, 0, 0, 0, 0, 0, 1]
    assert dec.pat_get_state()["live"] == 0                               # the sweep leaves an empty batch
    dec.close()


def test_predictor_fitted_to_a_measured_grid_predicts_a_held_out_point():
    """The latency predictor (host C++) on rows this GPU just measured: lines reproduce their own
    points closely and a held-out (batch, length) point inside the grid is predicted to within 25 %."""
    shard = pi.CONFIGS["7b_tp1"]["shard"].with_layers(4)
    pat = _pat()
    dec = make_decoder(shard, 16, 2048 + 128, 16 * 2048 + 16 * 128)
    pat.load_synthetic_weights(dec, shard)
    rows = dec.pat_profile_grid([1, 16], [256, 1024, 2048], 1 << 16, steps=20, warmup=3, reps=2)
    assert all(r["skipped"] == 0 for r in rows)
    pred = pat.Predictor([(r["tp_degree"], r["batch"], r["sum_context"], r["mean_us"]) for r in rows])
    for r in rows:
        assert abs(pred.pat_predictor_query(1, r["batch"], r["sum_context"]) / r["mean_us"] - 1.0) < 0.10
    a1, b1 = pred.pat_predictor_line(1, 16)
    assert b1 > 0.0                                    # more context tokens cost more time
    held = dec.pat_profile_grid([4], [1024], 1 << 16, steps=20, warmup=3, reps=2)[0]
    p = pred.pat_predictor_query(1, 4, held["sum_context"])
    print(f"held-out B=4 L=1024: measured {held['mean_us']:.1f} us, predicted {p:.1f} us")
    assert abs(p / held["mean_us"] - 1.0) < 0.25
    dec.close()


@pytest.mark.parametrize("hq,hkv,tp,rank", [(4, 4, 2, 1), (4, 4, 4, 3), (8, 2, 4, 2), (8, 2, 4, 1)])
def test_weight_reslice_from_the_unsharded_layer_is_bitwise_the_shard(hq, hkv, tp, rank):
    """Loading a rank's layer by slicing the unsharded tensors on the fly (weight re-slice after a TP
    change) gives bit-for-bit the logits of loading the rank's own contiguous slices; the last two cases
    have fewer KV heads than ranks (replicated KV heads)."""
    m = pi.ModelShape(2, 256, hq, hkv, 64, 1024, 1024)
    shard, full = pi.shard_of(m, tp, rank), pi.shard_of(m, 1, 0)
    pat = _pat()
    req = pi.rollout_requests(shard, 5, (20, 90), steps=3)
    outs = []
    for sliced in (False, True):
        cfg = pat.make_cfg(shard, 8, 128, 1024, 16)
        dec = pat.Decoder(cfg, DEV)
        if sliced:
            for l in range(m.n_layers):
                dec.pat_load_layer_from_full(l, pi.layer_weights(full, l, device=DEV))
                torch.cuda.synchronize()
            fw = pi.final_weights(shard, device=DEV); fw["embed"] = pi.embedding_table(shard, device=DEV)
            dec.pat_load_final(fw)
            torch.cuda.synchronize()
        else:
            pat.load_synthetic_weights(dec, shard, DEV)
        pat.admit_synthetic(dec, shard, req, DEV)
        got = [_gpu_step(dec, 5, shard.vocab) for _ in range(2)]
        outs.append(got)
        dec.close()
    for (la, na, _), (lb, nb, _) in zip(*outs):
        assert np.array_equal(la.view(np.uint32), lb.view(np.uint32)) and np.array_equal(na, nb)
    odec = make_oracle_decoder(shard)                                 # and the slices are the oracle's shard
    oracle_admit(odec, shard, req, range(5), 3)
    for la, na, _ in outs[1]:
        ref_logits, ref_next, _ = odec.step()
        check_logits(la, ref_logits)
        assert np.array_equal(na, ref_next)


@pytest.mark.parametrize("hq,hkv,d,tp,rank", [(4, 4, 64, 1, 0), (8, 2, 128, 1, 0), (4, 4, 64, 2, 1)])
def test_model_family_with_per_head_qk_norm(hq, hkv, d, tp, rank):
    """The second model family of the paper's evaluation normalises every q and k head (RMSNorm over
    head_dim, shared gains) before the rotary embedding: plain projection + one small kernel."""
    m = pi.ModelShape(2, 256, hq, hkv, d, 512, 512, qk_norm=True)
    _rollout_parity(pi.shard_of(m, tp, rank), 4, (20, 200), [3, 3, 2, 3])


def test_per_head_qk_norm_at_live_batch_40_and_the_unsharded_loader():
    m = pi.ModelShape(2, 256, 8, 4, 64, 1024, 1024, qk_norm=True)
    shard = pi.shard_of(m, 2, 1)
    _sampled_rows_parity(shard, 40, (30, 150), [0, 15, 16, 39], steps=2)
    # the re-slice loader carries the gains too: same logits bit for bit
    pat = _pat()
    req = pi.rollout_requests(shard, 3, (20, 60), steps=3)
    outs = []
    for sliced in (False, True):
        dec = pat.Decoder(pat.make_cfg(shard, 4, 128, 512, 16), DEV)
        if sliced:
            full = pi.shard_of(m, 1, 0)
            for l in range(m.n_layers):
                dec.pat_load_layer_from_full(l, pi.layer_weights(full, l, device=DEV))
                torch.cuda.synchronize()
            fw = pi.final_weights(shard, device=DEV); fw["embed"] = pi.embedding_table(shard, device=DEV)
            dec.pat_load_final(fw)
            torch.cuda.synchronize()
        else:
            pat.load_synthetic_weights(dec, shard, DEV)
        pat.admit_synthetic(dec, shard, req, DEV)
        outs.append(_gpu_step(dec, 3, shard.vocab)[0])
        dec.close()
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


def test_optional_fused_layer_kernel_rollout_parity(monkeypatch):
    """The persistent layer kernel (one launch for merge, O, gate/up, down and the next QKV or the head, with
    device-wide barriers), which a decoder created under PAT_ENABLE_FUSED=1 takes for live batches <= 16: the same
    rollout parity as the default path, tokens bit-exact, through compaction down to one sequence."""
    monkeypatch.setenv("PAT_ENABLE_FUSED", "1")
    pat = _pat()
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    probe = make_decoder(shard, 4, 64, 400, 16)
    used = probe.pat_decode_uses_fused_kernel()
    probe.close()
    if not used:
        pytest.skip("the device cannot keep the fused kernel's workgroups resident")
    targets = [3, 1, 7, 3, 12, 1, 5, 9, 2, 12, 4]
    worst, steps = _rollout_parity(shard, len(targets), (1, 150), targets, page_tokens=16)
    assert steps == 12
    # grouped-query shard with 128-wide heads (the other merge / attention instantiation)
    _rollout_parity(pi.shard_of(pi.ModelShape(2, 256, 8, 1, 128, 512, 512), 1, 0), 5, (10, 300), [6, 2, 9, 4, 9])
