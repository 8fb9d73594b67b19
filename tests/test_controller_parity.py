"""Host C++ of the latency predictor and the switch decision (through the C ABI) against the
CPU oracle, on seeded synthetic grids with the shape of a profile sweep (TP 1..8, the batch
sizes 1..256, three to five context lengths per batch size, B*L <= T_cap)."""
import math

import numpy as np
import pytest

import paper_2605_23945_amd as pat
from oracle import pat_controller as oc

REL = 1e-9          # both sides work in float64; they differ in summation order only


def _sweep(rng, noise=0.0):
    rows = []
    for tp in (1, 2, 4, 8):
        w = 13.2e9 / tp / 5e12 * 1e6 + 300.0 * math.log2(2 * tp)            # weights + a communication-like term
        for b in (1, 2, 4, 8, 16, 32, 64, 128, 256):
            for L in (256, 1024, 4096, 16384, 65536):
                if b * L > 2 ** 20:
                    continue
                t = b * L
                us = w * (1 + 0.02 * math.log2(b)) + 40.0 * b / tp + t * 0.5 / tp * 0.16 + rng.normal(0, noise)
                rows.append((tp, b, t, us))
    return rows


def _close(a, b):
    return abs(a - b) <= REL * max(1.0, abs(a), abs(b))


def test_lines_and_queries_match_the_oracle():
    rng = np.random.default_rng(11)
    rows = _sweep(rng, noise=25.0)
    o, p = oc.Predictor(rows), pat.Predictor(rows)
    for (tp, b), (alpha, beta) in o.lines.items():
        a2, b2 = p.pat_predictor_line(tp, b)
        assert _close(alpha, a2) and abs(beta - b2) <= REL * abs(beta)
    for _ in range(2000):
        tp = int(rng.choice([1, 2, 4, 8]))
        b = int(rng.integers(1, 400))
        t = float(rng.uniform(0, 3e6))
        assert _close(o.query(tp, b, t), p.pat_predictor_query(tp, b, t))
    with pytest.raises(pat.PatError):
        p.pat_predictor_query(3, 4, 100.0)              # TP degree that was not profiled
    with pytest.raises(pat.PatError):
        p.pat_predictor_line(1, 3)                      # batch size that was not profiled
    with pytest.raises(pat.PatError):
        p.pat_predictor_query(1, 0, 100.0)


def test_skipped_rows_are_ignored():
    rows = (pat.pat_grid_row * 3)()
    for r, (b, t, us, sk) in zip(rows, [(4, 1000, 10.0, 0), (4, 2000, 20.0, 0), (4, 3000, 999.0, 1)]):
        r.tp_degree, r.batch, r.sum_context, r.mean_us, r.skipped = 1, b, t, us, sk
    p = pat.Predictor(rows)
    assert p.pat_predictor_line(1, 4) == pytest.approx((0.0, 0.01))


def test_eq_1_to_3_match_the_oracle():
    rng = np.random.default_rng(5)
    for _ in range(20):
        ls = [int(x) for x in rng.integers(1, 20000, int(rng.integers(1, 40)))]
        tp = int(rng.choice([1, 2, 4, 8]))
        assert _close(oc.kv_move_time(ls, 32, 4096, 2, tp, 48e9), pat.pat_kv_move_seconds(ls, 32, 4096, 2, tp, 48e9))
        assert _close(oc.rms_length(ls), pat.pat_rms_length(ls))


@pytest.mark.parametrize("with_prefill", [False, True])
def test_decisions_match_the_oracle(with_prefill):
    rng = np.random.default_rng(23 + with_prefill)
    rows = _sweep(rng, noise=10.0)
    o, p = oc.Predictor(rows), pat.Predictor(rows)
    prefill = None
    if with_prefill:
        prefill = [(tp, b, L, 0.4 * b * L / tp + 2e-5 * b * L * L / tp) for tp in (1, 2, 4, 8) for b in (1, 4, 16, 64)
                   for L in (512, 2048, 8192)]
    n_switch = 0
    for case in range(300):
        tp = int(rng.choice([1, 2, 4, 8]))
        tp_list = [int(x) for x in rng.permutation([1, 2, 4, 8])]
        dp = 8 // tp
        lens_per_group = [[int(x) for x in rng.integers(200, 12000, int(rng.integers(0, 6)))] for _ in range(dp)]
        if sum(len(g) for g in lens_per_group) == 0:
            lens_per_group[0] = [3000]
        groups = [(len(g), float(sum(g))) for g in lens_per_group]
        lengths = [x for g in lens_per_group for x in g]
        l_gen = int(rng.integers(0, 4000)); l_max = l_gen + int(rng.integers(0, 6000))
        fixed = {(a, b): (0.0 if a == b else float(rng.uniform(2e5, 4e6))) for a in tp_list for b in tp_list}
        net = float(rng.uniform(10e9, 60e9))
        ref = oc.decide(o, tp, tp_list, groups, l_max, l_gen, lengths, (32, 4096, 2), fixed, net, 8,
                        oc.PrefillTable(prefill) if prefill else None)
        got = p.pat_switch_decide(tp, tp_list, groups, l_max, l_gen, lengths, (32, 4096, 2), fixed, net, 8, prefill)
        assert _close(ref[2], got[2]) and _close(ref[3], got[3]), case
        for (c0, r0, s0, t0), (c1, r1, s1, t1) in zip(ref[4], got[4]):
            assert c0 == c1 and _close(r0, r1) and _close(s0, s1) and _close(t0, t1), (case, c0)
        # the integer outcome must agree unless two totals are equal to rounding (then either is valid)
        tot = sorted(t for _, _, _, t in ref[4])
        margin = min(tot[1] - tot[0], abs(ref[2] - ref[3])) if len(tot) > 1 else 1.0
        if margin > 1e-6 * max(1.0, ref[3]):
            assert ref[0] == got[0] and ref[1] == got[1], case
        n_switch += ref[0]
    assert 20 < n_switch < 280          # the cases exercise both outcomes


def test_bad_inputs_are_rejected():
    p = pat.Predictor([(1, 1, 1000, 10.0), (2, 1, 1000, 8.0)])
    ok = dict(tp=1, tp_list=[1, 2], groups=[(1, 1000.0)], l_max=10, l_gen=0, lengths=[1000], model=(2, 64, 2),
              fixed_us={}, net_bytes_per_s=1e9, n_gpus=2)
    p.pat_switch_decide(**ok)
    for bad in (dict(tp=4), dict(tp_list=[2]), dict(n_gpus=3), dict(net_bytes_per_s=0.0), dict(tp_list=[1, 8])):
        with pytest.raises(pat.PatError):
            p.pat_switch_decide(**{**ok, **bad})


def test_unmeasured_prefill_rows_do_not_change_decisions():
    """A raw table as pat_profile_prefill writes it (latency -1 for pairs over the token cap or not
    fitting) must give the decision of the table with those rows removed; the oracle says the same."""
    rng = np.random.default_rng(41)
    rows = _sweep(rng, noise=10.0)
    o, p = oc.Predictor(rows), pat.Predictor(rows)
    full = [(tp, b, L, 0.4 * b * L / tp + 2e-5 * b * L * L / tp) for tp in (1, 2, 4, 8) for b in (1, 4, 16, 64)
            for L in (512, 2048, 8192, 32768)]
    raw = [(tp, b, L, us if b * L <= 2 ** 17 else -1.0) for tp, b, L, us in full]       # the profiler's cap rule
    raw += [(8, 128, 512, -1.0)]                                                         # a batch with no measured row at all
    clean = [r for r in raw if r[3] >= 0]
    assert 0 < len(clean) < len(raw)
    n_recomp = 0
    for case in range(120):
        tp = int(rng.choice([1, 2, 4, 8]))
        tp_list = [1, 2, 4, 8]
        dp = 8 // tp
        lens_per_group = [[int(x) for x in rng.integers(200, 30000, int(rng.integers(1, 5)))] for _ in range(dp)]
        groups = [(len(g), float(sum(g))) for g in lens_per_group]
        lengths = [x for g in lens_per_group for x in g]
        fixed = {(a, b): (0.0 if a == b else float(rng.uniform(2e5, 4e6))) for a in tp_list for b in tp_list}
        net = float(rng.uniform(0.2e9, 5e9))                     # slow links: recomputation often the cheaper
        args = (tp, tp_list, groups, 9000, int(rng.integers(0, 8000)), lengths, (32, 4096, 2), fixed, net, 8)
        a = p.pat_switch_decide(*args, raw)
        b = p.pat_switch_decide(*args, clean)
        ref = oc.decide(o, *args[:3], *args[3:], oc.PrefillTable(raw))
        assert a == b, case
        assert all(s >= 0.0 for _, _, s, _ in a[4]), case        # no cost pulled below zero by a -1 row
        for (c0, r0, s0, t0), (c1, r1, s1, t1) in zip(ref[4], a[4]):
            assert c0 == c1 and _close(s0, s1) and _close(t0, t1), (case, c0)
        move = 1e6 * oc.kv_move_time(lengths, 32, 4096, 2, tp, net)
        n_recomp += any(c != tp and s < fixed[(tp, c)] + move * (1 - 1e-12) for c, _, s, _ in a[4])
    assert n_recomp > 20                                          # the recomputation branch was the minimum often enough
    with pytest.raises(pat.PatError):                             # a (tp, batch, length) measured twice
        p.pat_switch_decide(*args, clean + [clean[0]])
