"""The offline profiler's sampling plan (Sec. 4.1, "Offline Profiler") as the C-ABI library enumerates it.

What the paper fixes: TP degrees 1, 2, 4, 8; ten batch sizes within [1, 256]; context lengths from 8 up to 128K;
a point (B, L) survives only if B * L <= T_cap; more points per octave below 512 tokens than above.  The counts
below are worked out by hand from those rules and the ladder the header states, not by calling the enumerator.
"""
import pytest

import paper_2605_23945_amd as pat


def _by_tp(points):
    out = {}
    for tp, b, l in points:
        out.setdefault(tp, []).append((b, l))
    return out


def test_plan_of_the_papers_deployment_row_count_by_hand():
    # T_cap = 2^20, lengths to 128K.  Lengths: 8 * 2^i for i = 0..14 (15 values) and 12 * 2^i below 512 for
    # i = 0..5 (12 .. 384, 6 values): 21.  Per batch size the largest kept length is T_cap / B:
    #   B = 1, 2, 4, 8: all 21;  16: <= 65536 -> 20;  32: 19;  64: 18;  128: <= 8192 -> 17;
    #   192: <= 5461 -> up to 4096 -> 16;  256: <= 4096 -> 16.
    per_tp = 4 * 21 + 20 + 19 + 18 + 17 + 16 + 16
    assert per_tp == 190
    pts = pat.pat_profile_plan(8, 1 << 20, 128 * 1024)
    assert len(pts) == 4 * per_tp
    groups = _by_tp(pts)
    assert sorted(groups) == [1, 2, 4, 8]
    for tp in groups:
        assert len(groups[tp]) == per_tp
        assert groups[tp] == groups[1]                      # the same (B, L) set for every degree


def test_plan_batches_lengths_pruning_and_density():
    t_cap = 1 << 20
    pts = pat.pat_profile_plan(8, t_cap, 128 * 1024)
    bl = _by_tp(pts)[1]
    batches = sorted({b for b, _ in bl})
    lengths = sorted({l for _, l in bl})
    assert len(batches) == 10 and batches[0] == 1 and batches[-1] == 256
    assert lengths[0] == 8 and lengths[-1] == 128 * 1024
    assert all(b * l <= t_cap for b, l in bl)
    # nothing that satisfies the budget is missing: the plan is the full grid minus the pruned corner
    assert set(bl) == {(b, l) for b in batches for l in lengths if b * l <= t_cap}
    # the largest batch stops at 4096 tokens, the smallest reaches the end
    assert max(l for b, l in bl if b == 256) == 4096
    assert max(l for b, l in bl if b == 1) == 128 * 1024
    # two points per octave below 512, one from 512 on
    below = [l for l in lengths if l < 512]
    above = [l for l in lengths if l >= 512]
    assert len(below) == 12 and len(above) == 9
    assert all(above[i + 1] == 2 * above[i] for i in range(len(above) - 1))
    ratios = [below[i + 1] / below[i] for i in range(len(below) - 1)]
    assert max(ratios) <= 1.5 + 1e-12
    # order: tp, then batch, then length, ascending
    assert pts == sorted(pts)


def test_plan_follows_the_pool_limit_and_the_gpu_count():
    # a pool of 2^18 tokens whose sequences stop at 40000 tokens, four GPUs: degrees 1, 2, 4; lengths to 32768
    pts = pat.pat_profile_plan(4, 1 << 18, 40000)
    groups = _by_tp(pts)
    assert sorted(groups) == [1, 2, 4]
    lens = sorted({l for _, l in groups[1]})
    assert lens[-1] == 32768 and len(lens) == 12 + 7
    # B = 256 -> L <= 1024: 12 + 2 lengths; B = 1 -> all 19
    assert sum(1 for b, _ in groups[1] if b == 256) == 14
    assert sum(1 for b, _ in groups[1] if b == 1) == 19
    # a budget below the shortest length times the batch leaves only the batches that fit
    tiny = pat.pat_profile_plan(1, 64, 8)
    assert tiny == [(1, b, 8) for b in (1, 2, 4, 8)]


def test_plan_errors():
    for args in ((0, 1 << 20, 1024), (8, 7, 1024), (8, 1 << 20, 7)):
        with pytest.raises(pat.PatError) as e:
            pat.pat_profile_plan(*args)
        assert e.value.code == -1
    with pytest.raises(pat.PatError) as e:
        pat.pat_profile_plan(8, 1 << 20, 128 * 1024, capacity=10)
    assert e.value.code != 0 and "760" in str(e.value)
