"""Pins of the oracle's KV send buffer (`oracle.kv_extract`, the gather of the paper's KV migration,
Sec. 4.2 "All-Gather and Slice") against statements of the layout that do not go through it:
a decodable tag per element, torch's stack / cat / permute, and hand cases.  CPU only.

The plausible mistakes these catch: head and token strides swapped, K and V swapped, `head0` or
`layer0` dropped, slots concatenated in slot-index order instead of the order given, a padded (not
valid-only) token count.
"""
import numpy as np
import torch

import oracle
from oracle import OracleDecoder

NL, HKV, D = 3, 4, 4
LENS = [3, 0, 5, 2]          # slot 1 holds no token yet
CAP_EXTRA = 2                # rows past kv_len exist in the cache and must never be sent


def _tag(kvsel, slot, layer, tok, head, e):
    """A distinct 16-bit value per (K|V, slot, layer, token, head, feature)."""
    return ((((kvsel * len(LENS) + slot) * NL + layer) * (max(LENS) + CAP_EXTRA) + tok) * HKV + head) * D + e


def _decoder():
    od = OracleDecoder(None, (NL, 32, HKV, HKV, D, 64, 1e-6, 10000.0), None, None, None)
    for s, L in enumerate(LENS):
        od.admit(100 + s, 7, L, 9, [np.zeros((L, HKV, D), np.uint16)] * NL, [np.zeros((L, HKV, D), np.uint16)] * NL, CAP_EXTRA)
        for l in range(NL):
            for t in range(L + CAP_EXTRA):          # rows past L carry tags too: sending one would show
                for h in range(HKV):
                    for e in range(D):
                        od.kc[s][l][t, h, e] = _tag(0, s, l, t, h, e)
                        od.vc[s][l][t, h, e] = _tag(1, s, l, t, h, e)
    assert _tag(1, len(LENS) - 1, NL - 1, max(LENS) + CAP_EXTRA - 1, HKV - 1, D - 1) < 65536
    return od


def test_every_element_decodes_to_its_coordinates():
    od = _decoder()
    slots, layer0, n_layers, head0, n_heads = [2, 0, 3], 1, 2, 1, 3
    buf = oracle.kv_extract(od, slots, layer0, n_layers, head0, n_heads)
    owner = [(s, t) for s in slots for t in range(LENS[s])]           # buffer token -> (slot, token of that slot)
    assert buf.shape == (n_layers, 2, n_heads, len(owner), D) and buf.dtype == np.uint16
    for l in range(n_layers):
        for kvsel in range(2):
            for h in range(n_heads):
                for bt, (s, t) in enumerate(owner):
                    for e in range(D):
                        assert buf[l, kvsel, h, bt, e] == _tag(kvsel, s, layer0 + l, t, head0 + h, e)


def test_against_stack_cat_permute():
    od = _decoder()
    for slots, layer0, n_layers, head0, n_heads in (([0, 1, 2, 3], 0, NL, 0, HKV), ([3, 2], 2, 1, 2, 2), ([2], 0, 2, 3, 1)):
        want = []
        for l in range(layer0, layer0 + n_layers):
            per_kv = []
            for cache in (od.kc, od.vc):
                toks = torch.cat([torch.from_numpy(cache[s][l][:LENS[s]].astype(np.int32)) for s in slots], dim=0)   # [T, hkv, d]
                per_kv.append(toks.permute(1, 0, 2)[head0:head0 + n_heads])                                           # [heads, T, d]
            want.append(torch.stack(per_kv))
        want = torch.stack(want).numpy()
        got = oracle.kv_extract(od, slots, layer0, n_layers, head0, n_heads)
        assert got.shape == want.shape and np.array_equal(got.astype(np.int32), want)


def test_hand_cases():
    od = _decoder()
    # one slot, one head, one layer: the slot's tokens of that head, K then V
    b = oracle.kv_extract(od, [0], 1, 1, 2, 1)
    assert b.shape == (1, 2, 1, 3, D)
    for t in range(3):
        assert list(b[0, 0, 0, t]) == [_tag(0, 0, 1, t, 2, e) for e in range(D)]
        assert list(b[0, 1, 0, t]) == [_tag(1, 0, 1, t, 2, e) for e in range(D)]
    # slot order is the order given, not the slot index order
    fwd, rev = oracle.kv_extract(od, [0, 2], 0, 1, 0, 1), oracle.kv_extract(od, [2, 0], 0, 1, 0, 1)
    assert np.array_equal(fwd[..., :3, :], rev[..., 5:, :]) and np.array_equal(fwd[..., 3:, :], rev[..., :5, :])
    assert not np.array_equal(fwd, rev)
    # a slot without tokens contributes nothing; alone it gives an empty token axis
    assert np.array_equal(oracle.kv_extract(od, [0, 1, 2], 0, NL, 0, HKV), oracle.kv_extract(od, [0, 2], 0, NL, 0, HKV))
    assert oracle.kv_extract(od, [1], 0, NL, 0, HKV).shape == (NL, 2, HKV, 0, D)
    # head0 > 0: heads [head0, head0 + n) of the full extract
    full = oracle.kv_extract(od, [3, 0], 0, NL, 0, HKV)
    assert np.array_equal(oracle.kv_extract(od, [3, 0], 0, NL, 1, 2), full[:, :, 1:3])
    # concatenating two ranks' buffers along the head axis is the full-head buffer (what the all-gather returns)
    lo, hi = oracle.kv_extract(od, [3, 0], 0, NL, 0, 2), oracle.kv_extract(od, [3, 0], 0, NL, 2, 2)
    assert np.array_equal(np.concatenate([lo, hi], axis=2), full)
