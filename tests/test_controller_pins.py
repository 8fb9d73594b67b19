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
