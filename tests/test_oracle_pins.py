"""Pins of the CPU oracle against things other than itself: float64 library
routines (torch), closed forms, invariants and brute force.  CPU only.

Each group names the plausible mistake it is there to catch.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import pat_inputs as pi
from oracle import bits

torch.manual_seed(0)
RNG = np.random.default_rng(1234)


def bf16_bits_of(x_f32: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns through torch's conversion (RNE)."""
    return bits(torch.from_numpy(np.asarray(x_f32, np.float32)).to(torch.bfloat16))


def widen(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rand_bf16(shape, std=1.0):
    return bf16_bits_of(RNG.standard_normal(shape).astype(np.float32) * std)


# ---- bf16 conversions (a wrong rounding mode or a shifted exponent) -----------

def test_bf16_widen_all_patterns(orc):
    for b in list(range(0, 0x7F80, 257)) + [0x3F80, 0xBF80, 0x0001, 0x8001, 0x7F7F]:
        assert orc.bf16_to_real(b) == float(widen(np.array([b], np.uint16))[0])


def test_bf16_round_matches_library_on_float32_inputs(orc):
    x = RNG.standard_normal(4000).astype(np.float32) * np.float32(3.0)
    ref = bf16_bits_of(x)
    got = np.array([orc.real_to_bf16(float(v)) for v in x], np.uint16)
    assert np.array_equal(ref, got)


def test_bf16_round_ties_to_even_and_roundtrip(orc):
    assert orc.real_to_bf16(1.0 + 2.0 ** -8) == 0x3F80        # tie -> even (down)
    assert orc.real_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82    # tie -> even (up)
    assert orc.real_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81   # just above a tie: no double rounding
    assert orc.real_to_bf16(-1.0 - 2.0 ** -8 - 2.0 ** -40) == 0xBF81
    assert orc.real_to_bf16(0.0) == 0 and orc.real_to_bf16(-0.0) == 0x8000
    for b in range(0x0080, 0x7F80, 97):
        assert orc.real_to_bf16(orc.bf16_to_real(b)) == b


# ---- matvec (transposed operand, wrong leading dimension) ----------------------

def test_matvec_vs_float64_matmul(orc):
    w = rand_bf16((37, 53), 0.02)
    x = RNG.standard_normal(53)
    ref = torch.from_numpy(widen(w)) @ torch.from_numpy(x)
    np.testing.assert_allclose(orc.matvec(w, x), ref.numpy(), rtol=1e-13, atol=1e-15)


def test_matvec_one_hot_and_rect(orc):
    w = rand_bf16((5, 9))
    for k in range(9):
        e = np.zeros(9); e[k] = 1.0
        assert np.array_equal(orc.matvec(w, e), widen(w)[:, k])


# ---- RMSNorm, SiLU, softmax ---------------------------------------------------

def test_rmsnorm_vs_library(orc):
    x = RNG.standard_normal(96) * 3.0
    g = rand_bf16(96)
    ref = F.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(widen(g)), eps=1e-6)
    np.testing.assert_allclose(orc.rmsnorm(x, g, 1e-6), ref.numpy(), rtol=1e-13)


def test_rmsnorm_unit_rms_and_scale_invariance(orc):
    x = RNG.standard_normal(128)
    ones = bf16_bits_of(np.ones(128, np.float32))
    y = orc.rmsnorm(x, ones, 0.0)
    assert abs(math.sqrt(float(np.mean(y * y))) - 1.0) < 1e-14
    np.testing.assert_allclose(orc.rmsnorm(7.5 * x, ones, 0.0), y, rtol=1e-13)
    # eps sits inside the square root, added to the mean (not to the sum, not outside)
    z = orc.rmsnorm(np.full(4, 2.0), ones[:4], 5.0)
    np.testing.assert_allclose(z, np.full(4, 2.0 / 3.0), rtol=1e-14)


def test_silu(orc):
    assert orc.silu(0.0) == 0.0
    for z in (-8.0, -1.0, 0.3, 2.5, 20.0):
        assert abs(orc.silu(z) - float(F.silu(torch.tensor(z, dtype=torch.float64)))) < 1e-14


def test_softmax_properties(orc):
    s = RNG.standard_normal(33) * 4
    p = orc.softmax(s)
    assert abs(p.sum() - 1.0) < 1e-14
    np.testing.assert_allclose(p, torch.softmax(torch.from_numpy(s), 0).numpy(), rtol=1e-13)
    np.testing.assert_allclose(orc.softmax(s + 1000.0), p, rtol=1e-10)   # shift invariance, no overflow
    np.testing.assert_allclose(orc.softmax(np.full(7, 3.0)), np.full(7, 1 / 7), rtol=1e-15)


# ---- rotary embedding (pairing, exponent, direction of rotation) -----------------

def test_rope_closed_forms(orc):
    v = RNG.standard_normal(8)
    assert np.array_equal(orc.rope(v, 0, 10000.0), v)                    # position 0 is the identity
    r = orc.rope([1.0, 0.0], 1, 10000.0)                                # d = 2: plain rotation by 1 rad
    np.testing.assert_allclose(r, [0.5403023058681398, 0.8414709848078965], rtol=1e-15)
    r = orc.rope([0.0, 1.0], 1, 10000.0)
    np.testing.assert_allclose(r, [-0.8414709848078965, 0.5403023058681398], rtol=1e-15)
    # d = 4: element 1 pairs with element 3 (half split) at angle pos * base^(-2/4) = 3 * 0.01
    r = orc.rope([0.0, 1.0, 0.0, 0.0], 3, 10000.0)
    np.testing.assert_allclose(r, [0.0, math.cos(0.03), 0.0, math.sin(0.03)], rtol=1e-15, atol=0)
    # d = 8, j = 3: angle = pos * base^(-6/8)
    e = np.zeros(8); e[3] = 1.0
    r = orc.rope(e, 5, 10000.0)
    th = 5 * 10000.0 ** (-0.75)
    np.testing.assert_allclose(r[[3, 7]], [math.cos(th), math.sin(th)], rtol=1e-14)


def test_rope_vs_complex_multiplication_and_relative_position(orc):
    d, base = 16, 10000.0
    q, k = RNG.standard_normal(d), RNG.standard_normal(d)
    for pos in (1, 17, 4095):
        zc = torch.complex(torch.from_numpy(q[: d // 2]), torch.from_numpy(q[d // 2:]))
        ang = pos * base ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
        rot = zc * torch.polar(torch.ones(d // 2, dtype=torch.float64), ang)
        ref = np.concatenate([rot.real.numpy(), rot.imag.numpy()])
        got = orc.rope(q, pos, base)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
        assert abs(np.linalg.norm(got) - np.linalg.norm(q)) < 1e-13
    # <R_p q, R_t k> depends on p - t only
    a = float(orc.rope(q, 40, base) @ orc.rope(k, 33, base))
    b = float(orc.rope(q, 7, base) @ k)
    assert abs(a - b) < 1e-12


# ---- attention -----------------------------------------------------------------

def test_attend_vs_library_sdpa(orc):
    n, d = 29, 16
    q = RNG.standard_normal(d)
    kb, vb = rand_bf16((n, d)), rand_bf16((n, d))
    o, p = orc.attend(q, kb, vb)
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None, None, None, :],
                                         torch.from_numpy(widen(kb))[None, None],
                                         torch.from_numpy(widen(vb))[None, None])
    np.testing.assert_allclose(o, ref[0, 0, 0].numpy(), rtol=1e-12, atol=1e-14)
    assert abs(p.sum() - 1.0) < 1e-14


def test_attend_special_cases(orc):
    d = 8
    q = RNG.standard_normal(d)
    kb, vb = rand_bf16((1, d)), rand_bf16((1, d))
    o, p = orc.attend(q, kb, vb)
    assert np.array_equal(o, widen(vb)[0]) and p[0] == 1.0          # length-1 cache returns V
    n = 12
    vb = rand_bf16((n, d))
    kb = np.repeat(rand_bf16((1, d)), n, 0)                         # identical keys -> mean of V
    o, _ = orc.attend(q, kb, vb)
    np.testing.assert_allclose(o, widen(vb).mean(0), rtol=1e-13, atol=1e-15)
    kb = rand_bf16((n, d))
    o0, _ = orc.attend(np.zeros(d), kb, vb)                          # q = 0 -> mean of V
    np.testing.assert_allclose(o0, widen(vb).mean(0), rtol=1e-13, atol=1e-15)
    o1, _ = orc.attend(q, kb, vb)
    perm = RNG.permutation(n)
    o2, _ = orc.attend(q, kb[perm], vb[perm])                        # joint permutation of (K, V)
    np.testing.assert_allclose(o1, o2, rtol=1e-12, atol=1e-14)


# ---- sub-layers against a float64 composition of library routines -----------------

def _torch_rope(x, pos, base):
    d = x.shape[-1]
    zc = torch.complex(x[..., : d // 2], x[..., d // 2:])
    ang = pos * base ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    r = zc * torch.polar(torch.ones(d // 2, dtype=torch.float64), ang)
    return torch.cat([r.real, r.imag], -1)


def _w64(b):
    return torch.from_numpy(widen(b))


def _torch_attn_sublayer(H, hq, hkv, d, eps, base, w, x, kc, vc, L):
    x = torch.from_numpy(x)
    h = F.rms_norm(x, (H,), _w64(w["g1"]), eps=eps)
    qkv = _w64(w["wqkv"]) @ h
    q, k = qkv[: hq * d].view(hq, d), qkv[hq * d:(hq + hkv) * d].view(hkv, d)
    if "gq" in w:                                            # per-head normalisation before the rotation
        q = F.rms_norm(q, (d,), _w64(w["gq"]), eps=eps)
        k = F.rms_norm(k, (d,), _w64(w["gk"]), eps=eps)
    q = _torch_rope(q, L, base)
    k = _torch_rope(k, L, base)
    v = qkv[(hq + hkv) * d:].view(hkv, d)
    kb = bits(k.to(torch.float32).to(torch.bfloat16)); vb = bits(v.to(torch.float32).to(torch.bfloat16))
    K = torch.cat([_w64(kc[:L]), _w64(kb)[None]], 0)       # [L+1, hkv, d]
    V = torch.cat([_w64(vc[:L]), _w64(vb)[None]], 0)
    o = F.scaled_dot_product_attention(q[None, :, None, :], K.permute(1, 0, 2)[None], V.permute(1, 0, 2)[None],
                                       enable_gqa=True)
    return (_w64(w["wo"]) @ o.reshape(-1)).numpy(), kb, vb


@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 2), (8, 1)])
def test_attn_sublayer_vs_library_composition(orc, hq, hkv):
    H, d, L, eps, base = 64, 16, 21, 1e-6, 10000.0
    w = dict(g1=bf16_bits_of(1 + 0.02 * RNG.standard_normal(H).astype(np.float32)),
             wqkv=rand_bf16(((hq + 2 * hkv) * d, H), 0.05), wo=rand_bf16((H, hq * d), 0.05))
    x = RNG.standard_normal(H)
    kc = np.zeros((L + 1, hkv, d), np.uint16); vc = np.zeros((L + 1, hkv, d), np.uint16)
    kc[:L] = rand_bf16((L, hkv, d)); vc[:L] = rand_bf16((L, hkv, d))
    ref, kb, vb = _torch_attn_sublayer(H, hq, hkv, d, eps, base, w, x, kc, vc, L)
    got = orc.attn_sublayer((H, hq, hkv, d, eps, base), w, x, kc, vc, L)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)
    # the appended entries are the bf16 roundings of k (rotated at position L) and v
    assert np.array_equal(kc[L], kb) and np.array_equal(vc[L], vb)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_attn_sublayer_with_per_head_qk_norm_vs_library_composition(orc, hq, hkv):
    H, d, L, eps, base = 64, 16, 13, 1e-6, 10000.0
    w = dict(g1=bf16_bits_of(1 + 0.02 * RNG.standard_normal(H).astype(np.float32)),
             wqkv=rand_bf16(((hq + 2 * hkv) * d, H), 0.05), wo=rand_bf16((H, hq * d), 0.05),
             gq=bf16_bits_of(1 + 0.3 * RNG.standard_normal(d).astype(np.float32)),
             gk=bf16_bits_of(1 + 0.3 * RNG.standard_normal(d).astype(np.float32)))
    x = RNG.standard_normal(H)
    kc = np.zeros((L + 1, hkv, d), np.uint16); vc = np.zeros((L + 1, hkv, d), np.uint16)
    kc[:L] = rand_bf16((L, hkv, d)); vc[:L] = rand_bf16((L, hkv, d))
    kc2, vc2 = kc.copy(), vc.copy()
    ref, kb, vb = _torch_attn_sublayer(H, hq, hkv, d, eps, base, w, x, kc, vc, L)
    got = orc.attn_sublayer((H, hq, hkv, d, eps, base), w, x, kc, vc, L)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)
    assert np.array_equal(kc[L], kb) and np.array_equal(vc[L], vb)
    # the normalisation matters (it is not a no-op on these inputs) and leaves v alone
    plain = orc.attn_sublayer((H, hq, hkv, d, eps, base), {k: v for k, v in w.items() if k not in ("gq", "gk")}, x, kc2, vc2, L)
    assert np.max(np.abs(plain - got)) > 1e-3 * np.max(np.abs(got))
    assert np.array_equal(vc2[L], vc[L]) and not np.array_equal(kc2[L], kc[L])
    # scale invariance: a normalised k does not change when the k rows of the projection are scaled
    w2 = dict(w); wq2 = widen(w["wqkv"]).astype(np.float32).copy(); wq2[hq * d:(hq + hkv) * d] *= 2.0; w2["wqkv"] = bf16_bits_of(wq2)
    kc3, vc3 = kc2.copy(), vc2.copy()
    got2 = orc.attn_sublayer((H, hq, hkv, d, eps, base), w2, x, kc3, vc3, L)
    np.testing.assert_allclose(got2, got, rtol=1e-6, atol=1e-9)


def test_ffn_sublayer_vs_library_composition(orc):
    H, Fd, eps = 48, 80, 1e-6
    w = dict(g2=bf16_bits_of(1 + 0.02 * RNG.standard_normal(H).astype(np.float32)),
             wg=rand_bf16((Fd, H), 0.2), wu=rand_bf16((Fd, H), 0.2), wd=rand_bf16((H, Fd), 0.2))
    x = RNG.standard_normal(H)
    h = F.rms_norm(torch.from_numpy(x), (H,), _w64(w["g2"]), eps=eps)
    ref = _w64(w["wd"]) @ (F.silu(_w64(w["wg"]) @ h) * (_w64(w["wu"]) @ h))
    np.testing.assert_allclose(orc.ffn_sublayer(H, Fd, eps, w, x), ref.numpy(), rtol=1e-11, atol=1e-13)
    w0 = dict(w, wg=np.zeros_like(w["wg"]))                       # zero gate -> the FFN adds nothing
    assert np.all(orc.ffn_sublayer(H, Fd, eps, w0, x) == 0.0)


# ---- tensor-parallel shards add up to the unsharded layer -----------------------

def _np_w(w):
    return {k: bits(v) for k, v in w.items()}


@pytest.mark.parametrize("tp", [2, 4])
def test_shard_partials_sum_to_unsharded(orc, tp):
    full = pi.CONFIGS["tiny_tp1"]["shard"]
    m = full.model
    H, d, eps, base, L = m.hidden, m.head_dim, m.rms_eps, m.rope_base, 9
    x = RNG.standard_normal(H)
    wf = _np_w(pi.layer_weights(full, 1))
    kf, vf = pi.kv_prefix(full, 5, 1, L)
    kc = np.zeros((L + 1, m.n_kv_heads, d), np.uint16); vc = np.zeros_like(kc)
    kc[:L], vc[:L] = bits(kf), bits(vf)
    ref_a = orc.attn_sublayer((H, m.n_q_heads, m.n_kv_heads, d, eps, base), wf, x, kc, vc, L)
    ref_f = orc.ffn_sublayer(H, m.ffn, eps, wf, x)
    sum_a, sum_f = np.zeros(H), np.zeros(H)
    for r in range(tp):
        s = pi.shard_of(m, tp, r)
        w = _np_w(pi.layer_weights(s, 1))
        ks, vs = pi.kv_prefix(s, 5, 1, L)
        kcs = np.zeros((L + 1, s.hkv, d), np.uint16); vcs = np.zeros_like(kcs)
        kcs[:L], vcs[:L] = bits(ks), bits(vs)
        sum_a += orc.attn_sublayer((H, s.hq, s.hkv, d, eps, base), w, x, kcs, vcs, L)
        sum_f += orc.ffn_sublayer(H, s.ffn, eps, w, x)
        # the shard's appended k, v are the shard's heads of the unsharded append
        assert np.array_equal(kcs[L], kc[L, r * s.hkv:(r + 1) * s.hkv])
    np.testing.assert_allclose(sum_a, ref_a, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(sum_f, ref_f, rtol=1e-11, atol=1e-14)


def test_vocab_shards_concatenate_and_global_argmax(orc):
    full = pi.CONFIGS["tiny_tp1"]["shard"]
    m = full.model
    x = RNG.standard_normal(m.hidden)
    ref = orc.logits(m.hidden, m.rms_eps, _np_w(pi.final_weights(full)), x)
    parts, best = [], (-np.inf, -1)
    for r in range(4):
        s = pi.shard_of(m, 4, r)
        lg = orc.logits(m.hidden, m.rms_eps, _np_w(pi.final_weights(s)), x)
        parts.append(lg)
        j = orc.argmax(lg)
        if lg[j] > best[0]:
            best = (lg[j], r * s.vocab + j)
    assert np.array_equal(np.concatenate(parts), ref)
    assert best[1] == orc.argmax(ref)


# ---- whole step ---------------------------------------------------------------------

def _tiny_decoder(orc, shard, zero_out=False, n_seq=3, steps=4):
    from oracle import OracleDecoder
    m = shard.model
    lw = [_np_w(pi.layer_weights(shard, l)) for l in range(m.n_layers)]
    if zero_out:
        for w in lw:
            w["wo"] = np.zeros_like(w["wo"]); w["wd"] = np.zeros_like(w["wd"])
    fw = _np_w(pi.final_weights(shard))
    emb = bits(pi.embedding_table(shard))
    dec = OracleDecoder(orc, (m.n_layers, m.hidden, shard.hq, shard.hkv, m.head_dim, shard.ffn, m.rms_eps,
                              m.rope_base), lambda l: lw[l], fw, lambda t: emb[t], vocab0=shard.rank * shard.vocab)
    req = pi.rollout_requests(shard, n_seq, (5, 20), steps=steps)
    for i in range(n_seq):
        kv = [pi.kv_prefix(shard, i, l, int(req["kv_len"][i])) for l in range(m.n_layers)]
        dec.admit(i, req["token"][i], req["kv_len"][i], req["target"][i],
                  [bits(a) for a, _ in kv], [bits(b) for _, b in kv], steps + 1)
    return dec, req, emb, fw


def test_step_closed_form_with_zero_output_projections(orc):
    """Wo = Wd = 0 leaves the residual equal to the embedding: logits = RMSNorm(E[tok]) Wlm^T."""
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    m = shard.model
    dec, req, emb, fw = _tiny_decoder(orc, shard, zero_out=True)
    logits, nxt, _ = dec.step()
    for i in range(3):
        e = _w64(emb[int(req["token"][i])])
        ref = _w64(fw["wlm"]) @ F.rms_norm(e, (m.hidden,), _w64(fw["gf"]), eps=m.rms_eps)
        np.testing.assert_allclose(logits[i], ref.numpy(), rtol=1e-11, atol=1e-14)
        assert nxt[i] == int(torch.argmax(ref))
    assert np.array_equal(dec.kv_len, req["kv_len"] + 1) and np.all(dec.gen == 1)


def test_step_rows_are_independent_and_f32_twin_agrees(orc, orc32):
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    d3, _, _, _ = _tiny_decoder(orc, shard, n_seq=3)
    d1, _, _, _ = _tiny_decoder(orc, shard, n_seq=1)
    l3, n3, _ = d3.step()
    l1, n1, _ = d1.step()
    assert np.array_equal(l3[0], l1[0]) and n3[0] == n1[0]       # row 0 does not see rows 1, 2
    d32, _, _, _ = _tiny_decoder(orc32, shard, n_seq=3)
    l32, n32, _ = d32.step()
    scale = l3.std()
    assert np.max(np.abs(l32 - l3)) < 1e-4 * scale               # the oracle's own rounding is far below tolerance
    assert np.array_equal(n32, n3)


def test_golden_tiny_rollout(orc):
    """The stored tokens and logits were written by tests/golden/make_tiny_golden.py (oracle only)."""
    import json, os
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_tp1_rollout.json")
    gold = json.load(open(path))
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    dec, _, _, _ = _tiny_decoder(orc, shard, n_seq=gold["n_seq"], steps=gold["steps"])
    for s in range(gold["steps"]):
        logits, nxt, _ = dec.step()
        assert nxt.tolist() == gold["tokens"][s]
        np.testing.assert_allclose(logits[0, :8], gold["logits_row0_first8"][s], rtol=1e-9, atol=1e-12)


# ---- argmax, finish flags, compaction ----------------------------------------------

def test_argmax_rules(orc):
    v = np.zeros(50, np.float32); v[17] = 3.0
    assert orc.argmax_f32(v) == 17 and orc.argmax(v.astype(np.float64)) == 17
    v[40] = 3.0; v[9] = 3.0
    assert orc.argmax_f32(v) == 9                                   # lowest index among equal maxima
    v[3] = np.nan
    assert orc.argmax_f32(v) == 9                                   # NaN never wins
    v[:] = -np.inf
    assert orc.argmax_f32(v) == 0
    v[30] = -1e30
    assert orc.argmax_f32(v) == 30
    v[45] = np.inf
    assert orc.argmax_f32(v) == 45
    x = RNG.standard_normal(1000).astype(np.float32)
    assert orc.argmax_f32(x) == int(np.argmax(x))


def test_finish_and_compaction_brute_force(orc):
    for trial in range(40):
        B = int(RNG.integers(0, 20))
        tok = RNG.integers(0, 6, B).astype(np.int32)
        gen = RNG.integers(0, 5, B).astype(np.int32); kv = RNG.integers(1, 50, B).astype(np.int32)
        target = RNG.integers(1, 6, B).astype(np.int32)
        eos = int(RNG.integers(-1, 6))
        g0, k0 = gen.copy(), kv.copy()
        fin, nf = orc.finish(tok, gen, kv, target, eos)
        assert np.array_equal(gen, g0 + 1) and np.array_equal(kv, k0 + 1)
        ref = (g0 + 1 >= target) | ((tok == eos) if eos >= 0 else np.zeros(B, bool))
        assert np.array_equal(fin.astype(bool), ref) and nf == int(ref.sum())
        m, nb = orc.compact_map(fin)
        survivors = np.flatnonzero(~ref)
        assert nb == len(survivors)
        assert np.array_equal(m[survivors], np.arange(nb)) and np.all(m[ref] == -1)
    for mask in ([0, 0, 0], [1, 1, 1], [1, 0, 1, 0, 1], [0, 1, 1], [1, 1, 0], []):
        m, nb = orc.compact_map(np.array(mask, np.int32))
        assert nb == mask.count(0)


def test_decoder_compaction_preserves_survivors(orc):
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    dec, req, _, _ = _tiny_decoder(orc, shard, n_seq=3, steps=4)
    dec.target[:] = [1, 3, 1]                                       # slots 0 and 2 finish after one step
    _, nxt, nf = dec.step()
    assert nf == 2 and dec.fin.tolist() == [1, 0, 1]
    k_before = dec.kc[1][0].copy()
    assert dec.compact() == 1
    assert dec.seq_id.tolist() == [1] and dec.tok.tolist() == [int(nxt[1])]
    assert dec.kv_len.tolist() == [int(req["kv_len"][1]) + 1] and np.array_equal(dec.kc[0][0], k_before)
    # compact-then-step equals stepping a batch that only ever held the survivor
    solo, _, _, _ = _tiny_decoder(orc, shard, n_seq=3, steps=4)
    solo.target[:] = [1, 3, 1]
    for name in ("seq_id", "tok", "kv_len", "gen", "target", "fin"):
        setattr(solo, name, getattr(solo, name)[[1]].copy())
    solo.kc, solo.vc = [solo.kc[1]], [solo.vc[1]]
    solo.step()
    la, na, _ = dec.step()
    lb, nb_, _ = solo.step()
    assert np.array_equal(la, lb) and np.array_equal(na, nb_)


# ---- prefill (an off-by-one in the causal window, a rotation at the wrong position) ----------

def _torch_prefill(shard, lw, emb, tokens):
    """All positions of one sequence at once, as matrices with the library's causal mask: K/V bits
    [layer][T, hkv, d] of the whole sequence."""
    m = shard.model
    H, hq, hkv, d = m.hidden, shard.hq, shard.hkv, m.head_dim
    T = len(tokens)
    X = torch.stack([_w64(emb[int(t)]) for t in tokens])                       # [T, H]
    pos = torch.arange(T, dtype=torch.float64)
    inv = m.rope_base ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    rot = torch.polar(torch.ones(T, d // 2, dtype=torch.float64), pos[:, None] * inv[None])   # [T, d/2]

    def rope(a):                                                               # [T, heads, d]
        z = torch.complex(a[..., : d // 2], a[..., d // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    ks, vs = [], []
    for w in lw:
        h = F.rms_norm(X, (H,), _w64(w["g1"]), eps=m.rms_eps)
        qkv = h @ _w64(w["wqkv"]).T
        q = rope(qkv[:, : hq * d].reshape(T, hq, d))
        k = rope(qkv[:, hq * d:(hq + hkv) * d].reshape(T, hkv, d))
        v = qkv[:, (hq + hkv) * d:].reshape(T, hkv, d)
        kb = bits(k.to(torch.float32).to(torch.bfloat16)); vb = bits(v.to(torch.float32).to(torch.bfloat16))
        ks.append(kb); vs.append(vb)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], _w64(kb).permute(1, 0, 2)[None],
                                           _w64(vb).permute(1, 0, 2)[None], is_causal=True, enable_gqa=True)
        X = X + o[0].permute(1, 0, 2).reshape(T, hq * d) @ _w64(w["wo"]).T
        h = F.rms_norm(X, (H,), _w64(w["g2"]), eps=m.rms_eps)
        X = X + (F.silu(h @ _w64(w["wg"]).T) * (h @ _w64(w["wu"]).T)) @ _w64(w["wd"]).T
    return ks, vs


def test_prefill_vs_whole_sequence_causal_attention_of_the_library(orc):
    """The oracle's token-by-token prefill against the matrix form with a causal mask.  Layer 2's
    K/V depend on layer 1's attention output at every position, so a window that is one position
    short or long, or a rotation by the wrong position, changes them."""
    from oracle import prefill
    shard = pi.CONFIGS["tiny_tp1"]["shard"]
    m = shard.model
    dec, req, emb, fw = _tiny_decoder(orc, shard, n_seq=2)
    lw = [dec.layer_w(l) for l in range(m.n_layers)]
    for slot in range(2):
        T = int(dec.kv_len[slot])
        toks = RNG.integers(0, shard.vocab, T)
        before = [dec.kc[slot][l].copy() for l in range(m.n_layers)]
        prefill(dec, slot, toks)
        ks, vs = _torch_prefill(shard, lw, emb, toks)
        for l in range(m.n_layers):
            assert not np.array_equal(dec.kc[slot][l][:T], before[l][:T])       # the synthetic prefix was replaced
            assert np.array_equal(dec.kc[slot][l][:T], ks[l]), f"K layer {l}"
            assert np.array_equal(dec.vc[slot][l][:T], vs[l]), f"V layer {l}"
            assert np.array_equal(dec.kc[slot][l][T:], before[l][T:])           # nothing written past the sequence
    # the slots' step state is untouched and the next step runs from the rebuilt cache
    assert np.array_equal(dec.kv_len, req["kv_len"]) and np.all(dec.gen == 0)
    dec.step()
    assert np.array_equal(dec.kv_len, req["kv_len"] + 1)
