"""Host logic of bench.py that needs no GPU: the rollout's step histogram (arithmetic on the request table) against a
step-by-step simulation, the bucket table, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def _simulate(kv_len, target):
    """Decode until every sequence has produced `target` tokens: live batch before each step, context tokens after it."""
    kv, gen = kv_len.astype(np.int64).copy(), np.zeros(len(kv_len), np.int64)
    alive = np.ones(len(kv_len), bool)
    live, peak = [], 0
    while alive.any():
        live.append(int(alive.sum()))
        kv[alive] += 1; gen[alive] += 1
        peak = max(peak, int(kv[alive].sum()))
        alive &= gen < target
    return live, peak


def test_rollout_plan_matches_a_step_by_step_simulation():
    rng = np.random.default_rng(5)
    for n in (1, 7, 40):
        req = {"kv_len": rng.integers(1, 50, n).astype(np.int32), "target": rng.integers(1, 30, n).astype(np.int32)}
        steps, live, peak = bench.rollout_plan(req)
        sim_live, sim_peak = _simulate(req["kv_len"], req["target"])
        assert steps == len(sim_live) == int(req["target"].max())
        assert live.tolist() == sim_live
        assert peak == sim_peak
        assert int(live.sum()) == int(req["target"].sum())          # every sequence produces exactly its target


def test_buckets_partition_the_live_batch_range():
    names = [bench.bucket_name(lo, hi) for lo, hi in bench.BUCKETS]
    assert names[:5] == ["1", "2", "3-4", "5-8", "9-16"] and "129-256" in names
    covered = []
    for lo, hi in bench.BUCKETS:
        covered += list(range(lo, hi + 1))
    assert covered == list(range(1, bench.BUCKETS[-1][1] + 1))       # no gap, no overlap
    # weighting: the buckets' step counts add up to the rollout's steps
    live = np.array([5, 5, 4, 4, 4, 2, 1, 1, 1, 1])
    per_bucket = [int(((live >= lo) & (live <= hi)).sum()) for lo, hi in bench.BUCKETS]
    assert sum(per_bucket) == len(live)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""
