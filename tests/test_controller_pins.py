"""Pins of the controller oracle (latency predictor, Algorithm 1, Eq. (1)-(4)) against things
other than itself: exact lines, closed forms, hand-computed numbers, brute force."""
import itertools
import math

import numpy as np
import pytest

from oracle import pat_controller as oc


def _grid(lines, ts):
    """rows of points lying exactly on given (tp, batch) -> (alpha, beta) lines"""
    return [(tp, b, t, a + be * t) for (tp, b), (a, be) in lines.items() for t in ts]


def test_fit_line_against_numpy_polyfit_and_exact_cases():
    rng = np.random.default_rng(7)
    t = rng.uniform(1e3, 1e6, 12)
    y = 800.0 + 3.5e-3 * t + rng.normal(0, 5.0, 12)
    a, b = oc.fit_line(list(t), list(y))
    pb, pa = np.polyfit(t, y, 1)                       # library routine, different algorithm (SVD)
    assert abs(a - pa) <= 1e-6 * abs(pa) and abs(b - pb) <= 1e-9 * abs(pb)
    assert oc.fit_line([2.0, 4.0], [10.0, 20.0]) == pytest.approx((0.0, 5.0))   # two points: the chord
    assert oc.fit_line([5.0], [42.0]) == (42.0, 0.0)
    assert oc.fit_line([3.0, 3.0, 3.0], [1.0, 2.0, 6.0]) == (3.0, 0.0)          # no spread in T: the mean
    # residuals of a least-squares line are orthogonal to 1 and to t
    r = y - (a + b * t)
    assert abs(r.sum()) <= 1e-6 and abs((r * t).sum()) <= 1e-1


def test_query_reproduces_lines_and_interpolates_along_batch():
    lines = {(1, 1): (1000.0, 1e-3), (1, 4): (1300.0, 2e-3), (1, 16): (2000.0, 5e-3), (4, 1): (400.0, 5e-4)}
    p = oc.Predictor(_grid(lines, [1e3, 5e4, 2e5]))
    for (tp, b), (a, be) in lines.items():
        for t in (0.0, 777.0, 1e6):                                             # on and beyond the profiled T range
            assert p.query(tp, b, t) == pytest.approx(a + be * t, rel=1e-12)
    t = 4e4
    assert p.query(1, 10, t) == pytest.approx(0.5 * (1300 + 2e-3 * t) + 0.5 * (2000 + 5e-3 * t), rel=1e-12)
    assert p.query(1, 2, t) == pytest.approx((2 / 3) * (1000 + 1e-3 * t) + (1 / 3) * (1300 + 2e-3 * t), rel=1e-12)
    assert p.query(1, 64, t) == pytest.approx(2000 + 5e-3 * t, rel=1e-12)       # above the range: last line alone
    assert p.query(4, 9, t) == pytest.approx(400 + 5e-4 * t, rel=1e-12)         # one profiled batch size only


def test_est_rem_time_closed_forms():
    lines = {(2, 8): (500.0, 0.0), (2, 32): (900.0, 0.0)}
    p = oc.Predictor(_grid(lines, [1e3, 1e4]))
    assert oc.est_rem_time(p, 2, [(8, 5000.0)], 100, 40) == pytest.approx(60 * 500.0)           # constant latency
    assert oc.est_rem_time(p, 2, [(8, 5e3), (32, 1e3)], 100, 40) == pytest.approx(60 * 900.0)   # slowest group
    assert oc.est_rem_time(p, 2, [(8, 5e3)], 40, 40) == 0.0
    assert oc.est_rem_time(p, 2, [(0, 0.0)], 100, 40) == 0.0
    # linear in T: arithmetic series  n a + beta (n T + B n (n - 1) / 2)
    p2 = oc.Predictor(_grid({(1, 4): (100.0, 0.01)}, [0.0, 1e5]))
    n, b, t0 = 250, 4, 3000.0
    want = n * 100.0 + 0.01 * (n * t0 + b * n * (n - 1) / 2)
    assert oc.est_rem_time(p2, 1, [(b, t0)], 1000, 750) == pytest.approx(want, rel=1e-12)


def test_merged_batch_and_tokens():
    assert oc.compute_merged([(3, 300.0), (0, 0.0), (2, 500.0), (1, 100.0)], 8, 2) == (2, 225.0)   # 6 samples over 4 groups
    assert oc.compute_merged([(3, 300.0), (0, 0.0), (2, 500.0), (1, 100.0)], 8, 8) == (6, 900.0)   # one group
    assert oc.compute_merged([(5, 50.0)] * 8, 8, 1) == (5, 50.0)


def test_kv_move_time_hand_computed():
    # two samples of 1000 and 3000 tokens, 32 layers, hidden 4096, 2 bytes, source TP 2:
    # 2 * 32 * 4000 * 2048 * 2 = 1 048 576 000 bytes; at 50e9 B/s -> 20.97152 ms
    assert oc.kv_move_time([1000, 3000], 32, 4096, 2, 2, 50e9) == pytest.approx(0.02097152, rel=1e-12)
    assert oc.kv_move_time([], 32, 4096, 2, 2, 50e9) == 0.0


def test_rms_length_identity():
    ls = [100, 2000, 333, 4096, 7]
    r = oc.rms_length(ls)
    assert len(ls) * r * r == pytest.approx(sum(l * l for l in ls), rel=1e-12)
    assert oc.rms_length([512, 512]) == pytest.approx(512.0)
    assert r >= sum(ls) / len(ls)                                   # RMS is never below the mean


def test_prefill_table_lookup():
    rows = [(4, 2, 1000, 10.0), (4, 2, 2000, 30.0), (4, 2, 4000, 110.0), (4, 8, 1000, 40.0), (4, 8, 4000, 400.0)]
    pf = oc.PrefillTable(rows)
    assert pf.query(4, 2, 1500) == pytest.approx(20.0)
    assert pf.query(4, 2, 3000) == pytest.approx(70.0)
    assert pf.query(4, 2, 5000) == pytest.approx(150.0)             # last segment extended
    assert pf.query(4, 2, 500) == pytest.approx(0.0)                # first segment extended
    assert pf.query(4, 5, 1000) == pytest.approx(25.0)              # halfway between the batch sizes
    assert pf.query(4, 64, 2500) == pytest.approx(40.0 + 360.0 * 0.5)


def _toy():
    # per-step latency (us): TP1 is cheap at large batch, TP4 at small batch (weights dominate)
    lines = {(1, 1): (4000.0, 1e-3), (1, 64): (9000.0, 1e-3), (4, 1): (1500.0, 5e-4), (4, 64): (12000.0, 5e-4)}
    return oc.Predictor(_grid(lines, [1e3, 1e5]))


def test_algorithm_1_hand_computed_switch_and_no_switch():
    p = _toy()
    model = (32, 4096, 2)
    fixed = {(1, 4): 1.0e6, (1, 1): 0.0, (4, 1): 1.0e6, (4, 4): 0.0}
    # 4 GPUs at TP1 = 4 DP groups with one straggler each of 3000 tokens; 1000 steps to go
    groups = [(1, 3000.0)] * 4
    lengths = [3000] * 4
    do, tp_new, t_cur, t_best, totals = oc.decide(p, 1, [1, 4], groups, 4000, 3000, lengths, model, fixed, 25e9, 4)
    # current: sum_k 4000 + 1e-3 (3000 + k) = 1000*4003 + 1e-3*499500
    assert t_cur == pytest.approx(4003000.0 + 499.5)
    # TP4: one group of 4 samples, 12000 tokens: B = 4 between profiled 1 and 64: w = 3/63
    w = 3 / 63
    rem4 = sum((1 - w) * (1500 + 5e-4 * (12000 + 4 * k)) + w * (12000 + 5e-4 * (12000 + 4 * k)) for k in range(1000))
    move = 4 * 2 * 32 * 3000 * 4096 * 2 / 25e9 * 1e6           # source TP 1
    assert totals[1][1] == pytest.approx(rem4, rel=1e-12)
    assert totals[1][2] == pytest.approx(1.0e6 + move, rel=1e-12)
    assert do and tp_new == 4 and t_best == pytest.approx(rem4 + 1.0e6 + move, rel=1e-12)
    # ten times fewer steps left: the switch no longer pays for itself
    do2, tp2, t_cur2, t_best2, _ = oc.decide(p, 1, [1, 4], groups, 3100, 3000, lengths, model, fixed, 25e9, 4)
    assert not do2 and t_cur2 < 1.0e6
    # the current degree is itself a candidate: with all candidates dearer, tp_new stays
    assert tp2 == 1 and t_best2 == pytest.approx(t_cur2)


def test_algorithm_1_tie_keeps_current_and_first_minimum_wins():
    lines = {(1, 2): (100.0, 0.0), (2, 2): (100.0, 0.0), (4, 2): (100.0, 0.0), (2, 4): (100.0, 0.0), (4, 8): (100.0, 0.0),
             (1, 1): (100.0, 0.0), (2, 1): (100.0, 0.0), (4, 1): (100.0, 0.0)}
    p = oc.Predictor(_grid(lines, [1.0, 2.0]))
    zero = {(a, b): 0.0 for a in (1, 2, 4) for b in (1, 2, 4)}
    groups = [(2, 10.0)] * 4
    do, tp_new, t_cur, t_best, _ = oc.decide(p, 2, [4, 1, 2], groups, 10, 0, [], (1, 1, 1), zero, 1e9, 4)
    assert t_cur == t_best == 1000.0
    assert tp_new == 4 and not do                       # first of the equal candidates, but no strict gain


def test_algorithm_1_argmin_matches_brute_force():
    rng = np.random.default_rng(3)
    for _ in range(50):
        lines = {(tp, b): (float(rng.uniform(500, 5000)), float(rng.uniform(1e-4, 5e-3))) for tp in (1, 2, 4, 8) for b in (1, 8, 64)}
        p = oc.Predictor(_grid(lines, [1e3, 1e4, 1e5]))
        fixed = {(a, b): (0.0 if a == b else float(rng.uniform(1e5, 3e6))) for a in (1, 2, 4, 8) for b in (1, 2, 4, 8)}
        tp = int(rng.choice([1, 2, 4, 8]))
        dp = 8 // tp
        groups = [(int(rng.integers(0, 5)), 0.0) for _ in range(dp)]
        groups = [(b, float(b * rng.integers(500, 4000))) for b, _ in groups]
        if sum(b for b, _ in groups) == 0:
            continue
        lengths = [int(t / b) for b, t in groups for _ in range(b)]
        steps = int(rng.integers(10, 2000))
        do, tp_new, t_cur, t_best, totals = oc.decide(p, tp, [1, 2, 4, 8], groups, steps, 0, lengths, (32, 4096, 2), fixed, 40e9, 8)
        tot = [x[3] for x in totals]
        assert t_best == min(tot) and tp_new == [1, 2, 4, 8][int(np.argmin(tot))]
        assert do == (tp_new != tp and t_cur > t_best)
        for cand, t_rem, t_sw, _ in totals:
            assert (t_sw == 0.0) == (cand == tp)
            mb, mt = oc.compute_merged(groups, 8, cand)
            # remaining time is monotone in what it sums: never below steps x the cheapest step
            lo = min(p.query(cand, mb, mt), p.query(cand, mb, mt + (steps - 1) * mb))
            assert t_rem >= steps * lo * (1 - 1e-12)


# ---- T_switch with a prefill table: Eq. (3)-(4) and min(T_move, T_recomp) of Sec. 4.2 ----------------
# Mistakes these catch: the group batch of Eq. (4) taken as all samples instead of ceil(n / (G / tp')), the mean
# length instead of the RMS, the source degree's table instead of the target's, max instead of min, the fixed
# cost dropped or added twice, T_move in seconds added to microseconds.

def test_switch_cost_recomputation_branch_hand_computed():
    model = (32, 4096, 2)
    fixed = {(1, 4): 7000.0, (4, 1): 9000.0, (1, 2): 100.0, (1, 1): 0.0, (4, 4): 0.0}
    # target TP 4 on 8 GPUs: 2 DP groups; five unfinished samples -> ceil(5 / 2) = 3 per group
    lengths = [1000, 1000, 2000, 2000, 4000]
    l_rms = math.sqrt((2 * 1000 ** 2 + 2 * 2000 ** 2 + 4000 ** 2) / 5)          # 2280.35..., the mean is 2000
    assert l_rms == pytest.approx(2280.350850198276, rel=1e-15)
    rows = [(4, 2, 2000, 100.0), (4, 2, 3000, 200.0), (4, 4, 2000, 300.0), (4, 4, 3000, 500.0),
            (1, 3, 2000, 1.0), (1, 3, 3000, 2.0)]                                # TP 1 rows: the wrong table if used
    pf = oc.PrefillTable(rows)
    at2 = 100.0 + 100.0 * (l_rms - 2000) / 1000                                   # batch 2 curve at L_RMS
    at4 = 300.0 + 200.0 * (l_rms - 2000) / 1000                                   # batch 4 curve
    t_recomp = 0.5 * at2 + 0.5 * at4                                              # batch 3: halfway
    assert t_recomp == pytest.approx(200.0 + 150.0 * 0.280350850198276, rel=1e-12)
    # migration at 1 GB/s: 2 * 32 * 10000 tokens * 4096 / 1 * 2 bytes = 5.24288e9 bytes -> 5.24288 s = 5 242 880 us
    t_move_slow = 2 * 32 * 10000 * 4096 * 2 / 1e9 * 1e6
    assert t_move_slow == pytest.approx(5242880.0)
    # recomputation wins on a slow network
    got = oc.switch_cost_us(1, 4, lengths, model, fixed, 1e9, pf, 8)
    assert got == pytest.approx(7000.0 + t_recomp, rel=1e-12)
    # migration wins on a fast one: 1e15 B/s -> 5.24288 us
    got = oc.switch_cost_us(1, 4, lengths, model, fixed, 1e15, pf, 8)
    assert got == pytest.approx(7000.0 + 5.24288, rel=1e-12)
    # no table: migration whatever it costs; same degree: nothing
    assert oc.switch_cost_us(1, 4, lengths, model, fixed, 1e9, None, 8) == pytest.approx(7000.0 + t_move_slow, rel=1e-12)
    assert oc.switch_cost_us(4, 4, lengths, model, fixed, 1e9, pf, 8) == 0.0
    # a target degree the table holds no row for (TP 2): recomputation unavailable, not an error
    assert oc.switch_cost_us(1, 2, lengths, model, fixed, 1e9, pf, 8) == pytest.approx(100.0 + t_move_slow, rel=1e-12)
    # the source degree divides the migration volume (Eq. (1)): from TP 4 it is a quarter
    assert oc.switch_cost_us(4, 1, lengths, model, fixed, 1e9, None, 8) == pytest.approx(9000.0 + t_move_slow / 4, rel=1e-12)


def test_switch_cost_at_a_profiled_point_equals_the_table_entry():
    # equal lengths: L_RMS is that length; 8 samples onto TP 2 of 8 GPUs = 4 groups of 2: the (2, 2, 1024) entry itself
    pf = oc.PrefillTable([(2, 1, 1024, 11.0), (2, 2, 512, 17.0), (2, 2, 1024, 31.0), (2, 2, 2048, 77.0), (2, 4, 1024, 59.0)])
    fixed = {(8, 2): 5.0}
    assert oc.switch_cost_us(8, 2, [1024] * 8, (4, 256, 2), fixed, 1.0, pf, 8) == pytest.approx(5.0 + 31.0, rel=1e-15)
    # 7 samples still make groups of ceil(7 / 4) = 2; 9 samples make groups of 3: halfway between batch 2 and 4
    assert oc.switch_cost_us(8, 2, [1024] * 7, (4, 256, 2), fixed, 1.0, pf, 8) == pytest.approx(5.0 + 31.0, rel=1e-15)
    assert oc.switch_cost_us(8, 2, [1024] * 9, (4, 256, 2), fixed, 1.0, pf, 8) == pytest.approx(5.0 + 45.0, rel=1e-15)


def test_decide_with_prefill_table_recomputation_and_migration_outcomes():
    p = _toy()
    model = (32, 4096, 2)
    fixed = {(1, 4): 1.0e6, (1, 1): 0.0}
    groups, lengths = [(1, 3000.0)] * 4, [3000] * 4
    # 4 GPUs -> TP 4 is one group of all four samples at L_RMS = 3000: the (4, 4, 3000) entry
    pf = oc.PrefillTable([(4, 4, 3000, 250000.0), (4, 4, 6000, 900000.0)])
    move = 4 * 2 * 32 * 3000 * 4096 * 2 / 25e9 * 1e6                              # 251 658.24 us at 25 GB/s
    assert move == pytest.approx(251658.24)
    w = 3 / 63
    rem4 = sum((1 - w) * (1500 + 5e-4 * (12000 + 4 * k)) + w * (12000 + 5e-4 * (12000 + 4 * k)) for k in range(1000))
    do, tp_new, t_cur, t_best, totals = oc.decide(p, 1, [1, 4], groups, 4000, 3000, lengths, model, fixed, 25e9, 4, pf)
    assert totals[1][2] == pytest.approx(1.0e6 + 250000.0, rel=1e-12)             # recomputation is the cheaper by 1658 us
    assert do and tp_new == 4 and t_best == pytest.approx(rem4 + 1.0e6 + 250000.0, rel=1e-12)
    # a network twice as fast: migration (125 829.12 us) wins
    _, _, _, _, totals = oc.decide(p, 1, [1, 4], groups, 4000, 3000, lengths, model, fixed, 50e9, 4, pf)
    assert totals[1][2] == pytest.approx(1.0e6 + move / 2, rel=1e-12)
    # recomputation so cheap it flips a decision that migration alone loses: 100 steps left
    pf2 = oc.PrefillTable([(4, 4, 3000, 10.0)])
    slow = oc.decide(p, 1, [1, 4], groups, 3100, 3000, lengths, model, {(1, 4): 0.0, (1, 1): 0.0}, 1e6, 4, None)
    fast = oc.decide(p, 1, [1, 4], groups, 3100, 3000, lengths, model, {(1, 4): 0.0, (1, 1): 0.0}, 1e6, 4, pf2)
    assert not slow[0] and fast[0] and fast[1] == 4 and fast[4][1][2] == pytest.approx(10.0)


def test_prefill_table_ignores_unmeasured_rows_and_rejects_duplicates():
    rows = [(4, 2, 1000, 10.0), (4, 2, 2000, 30.0), (4, 2, 4000, 110.0)]
    marked = rows + [(4, 2, 3000, -1.0), (4, 2, 8000, -1.0), (4, 16, 1000, -1.0), (2, 2, 1000, float("nan"))]
    a, b = oc.PrefillTable(rows), oc.PrefillTable(marked)
    for L in (500, 1500, 3000, 3500, 9000):
        assert a.query(4, 2, L) == b.query(4, 2, L)
        assert a.query(4, 16, L) == b.query(4, 16, L)          # batch 16 had only an unmeasured row: no curve of its own
    assert b.query(4, 2, 3000) == pytest.approx(70.0)           # through the measured neighbours, not through -1
    assert b.query(2, 2, 1000) == math.inf                      # nothing measured for TP 2
    with pytest.raises(ValueError):
        oc.PrefillTable(rows + [(4, 2, 2000, 31.0)])
