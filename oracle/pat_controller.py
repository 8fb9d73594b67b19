"""CPU oracle of the latency predictor and the online switch decision (TEST INFRASTRUCTURE).

Plain float64 Python, loops written out.  Only tests, the smoke check and the CPU leg of the
benchmark may import this module; the product (the C++ in the HIP library) shares no code
with it.

What it follows (paper, Sec. 4.1 and 4.2):
  * "Online Latency Predictor": per (TP, profiled batch size) a straight line in the
    aggregate context tokens T fitted to the profiled points; a query (B, T) evaluates the
    lines of the two nearest profiled batch sizes and interpolates linearly along the batch
    dimension.
  * Algorithm 1 ("Online Switch Mechanism"): remaining decode time under the current TP
    degree, remaining time plus switch cost for every candidate, switch only if the best
    candidate differs from the current degree and is strictly cheaper.
  * Eq. (1), (2): KV migration time from the per-rank send volume; Eq. (3), (4):
    recomputation time as the profiled prefill latency at the RMS context length; the state
    handling cost is the smaller of the two.

Readings where the paper is silent (each also listed in the design notes):
  R1  est_rem_time sums the per-step latency over the L_max - L_gen steps that remain, with
      every unfinished sample running to L_max (the paper's conservative bound), so T grows
      by B per step: sum_k l(B, T + k B).  DP groups decode in lock step, the slowest group
      bounds the stage: the maximum over groups.
  R2  compute_merged_bs spreads the unfinished samples evenly over the G / tp' groups of the
      target layout: ceil(sum(rbs) / (G / tp')); the context tokens are spread the same way.
  R3  Outside the profiled batch range the nearest profiled batch size is used alone; the
      line is extended in T without clamping.  A batch size that was profiled is its own
      two neighbours.
  R4  Candidates are visited in list order and compared with strict "<", so the first of
      equally cheap candidates wins, and a tie with the current cost means no switch.
  R5  The profiled prefill latency is looked up like the decode latency: piecewise linear
      in L between profiled lengths (ends extended) at the two nearest batch sizes, then
      linear in B.  Without a prefill table recomputation is not available (infinite).
  R6  T_switch(tp, tp') = fixed[tp][tp'] + min(T_move, T_recomp) for tp' != tp, and 0 for
      tp' == tp; `fixed` (weight resharding, group updates, control overheads) is a measured
      input table.
"""
from __future__ import annotations

import math


def fit_line(ts, ys):
    """Least-squares line y = alpha + beta t through the points (normal equations).
    One point: a constant.  All t equal: a constant at the mean."""
    n = len(ts)
    if n == 0:
        raise ValueError("no points")
    mt = sum(ts) / n
    my = sum(ys) / n
    stt = sum((t - mt) * (t - mt) for t in ts)
    if n == 1 or stt == 0.0:
        return my, 0.0
    sty = sum((t - mt) * (y - my) for t, y in zip(ts, ys))
    beta = sty / stt
    return my - beta * mt, beta


class Predictor:
    """rows: iterable of (tp, batch, sum_context, mean_us) of measured grid points."""

    def __init__(self, rows):
        pts = {}
        for tp, b, t, us in rows:
            pts.setdefault((int(tp), int(b)), []).append((float(t), float(us)))
        self.lines = {}
        for key, p in pts.items():
            self.lines[key] = fit_line([q[0] for q in p], [q[1] for q in p])
        self.batches = {}
        for tp, b in self.lines:
            self.batches.setdefault(tp, []).append(b)
        for tp in self.batches:
            self.batches[tp].sort()

    def line_value(self, tp, b, t):
        alpha, beta = self.lines[(tp, b)]
        return alpha + beta * t

    def query(self, tp, batch, t):
        """Per-step latency l(B, T; TP) in microseconds."""
        bs = self.batches[tp]
        if batch <= bs[0]:
            return self.line_value(tp, bs[0], t)
        if batch >= bs[-1]:
            return self.line_value(tp, bs[-1], t)
        lo = max(b for b in bs if b <= batch)
        hi = min(b for b in bs if b >= batch)
        if lo == hi:
            return self.line_value(tp, lo, t)
        w = (batch - lo) / (hi - lo)
        return (1.0 - w) * self.line_value(tp, lo, t) + w * self.line_value(tp, hi, t)


def est_rem_time(pred, tp, groups, l_max, l_gen):
    """groups: list of (batch, context tokens) per DP group.  Microseconds (reading R1)."""
    steps = max(0, int(l_max) - int(l_gen))
    worst = 0.0
    for b, t in groups:
        if b <= 0:
            continue
        total = 0.0
        for k in range(steps):
            total += pred.query(tp, b, t + k * b)
        worst = max(worst, total)
    return worst


def compute_merged(groups, n_gpus, tp_new):
    """(batch, context tokens) of one DP group after redistribution (reading R2)."""
    dp = n_gpus // tp_new
    sb = sum(b for b, _ in groups)
    st = sum(t for _, t in groups)
    return -(-sb // dp), st / dp


def kv_move_time(lengths, n_layers, hidden, bytes_per_elem, tp_src, net_bytes_per_s):
    """Eq. (1), (2): seconds."""
    s = 0.0
    for li in lengths:
        s += 2.0 * n_layers * li * (hidden / tp_src) * bytes_per_elem
    return s / net_bytes_per_s


def rms_length(lengths):
    """Eq. (3)."""
    return math.sqrt(sum(float(l) * float(l) for l in lengths) / len(lengths))


class PrefillTable:
    """rows: (tp, batch, length, microseconds) of profiled prefill latencies (reading R5).

    Eq. (4) reads a PROFILED latency: a row whose latency is negative or NaN is how the profiler marks
    a (batch, length) pair it did not measure (over the token cap, or not fitting the pool) and is no
    point of any curve.  Two measured rows of one (tp, batch, length) are a malformed table."""

    def __init__(self, rows):
        self.curves = {}
        for tp, b, l, us in rows:
            if not (float(us) >= 0.0):              # unmeasured marker (-1) or NaN
                continue
            self.curves.setdefault((int(tp), int(b)), []).append((float(l), float(us)))
        for k in self.curves:
            self.curves[k].sort()
            ls = [q[0] for q in self.curves[k]]
            if len(set(ls)) != len(ls):
                raise ValueError(f"prefill table: length profiled twice for (tp, batch) = {k}")
        self.batches = {}
        for tp, b in self.curves:
            self.batches.setdefault(tp, []).append(b)
        for tp in self.batches:
            self.batches[tp].sort()

    def curve_value(self, tp, b, length):
        c = self.curves[(tp, b)]
        if len(c) == 1:
            return c[0][1]
        i = 0
        while i + 2 < len(c) and length > c[i + 1][0]:
            i += 1
        (l0, y0), (l1, y1) = c[i], c[i + 1]
        return y0 + (y1 - y0) * (length - l0) / (l1 - l0)

    def query(self, tp, batch, length):
        if tp not in self.batches:                  # nothing measured for this degree: recomputation unavailable
            return math.inf
        bs = self.batches[tp]
        if batch <= bs[0]:
            return self.curve_value(tp, bs[0], length)
        if batch >= bs[-1]:
            return self.curve_value(tp, bs[-1], length)
        lo = max(b for b in bs if b <= batch)
        hi = min(b for b in bs if b >= batch)
        if lo == hi:
            return self.curve_value(tp, lo, length)
        w = (batch - lo) / (hi - lo)
        return (1.0 - w) * self.curve_value(tp, lo, length) + w * self.curve_value(tp, hi, length)


def switch_cost_us(tp, tp_new, lengths, model, fixed_us, net_bytes_per_s, prefill, n_gpus):
    """T_switch in microseconds (reading R6).  model = (n_layers, hidden, bytes_per_elem)."""
    if tp_new == tp:
        return 0.0
    n_layers, hidden, bpe = model
    t_move = kv_move_time(lengths, n_layers, hidden, bpe, tp, net_bytes_per_s) * 1e6
    t_recomp = math.inf
    if prefill is not None and lengths:
        dp = n_gpus // tp_new
        b_group = -(-len(lengths) // dp)
        t_recomp = prefill.query(tp_new, b_group, rms_length(lengths))
    return fixed_us[(tp, tp_new)] + min(t_move, t_recomp)


def decide(pred, tp, tp_list, groups, l_max, l_gen, lengths, model, fixed_us, net_bytes_per_s, n_gpus,
           prefill=None):
    """One evaluation of Algorithm 1's loop body.  Returns (do_switch, tp_new, T_cur, T_best, totals)
    with times in microseconds and totals a list of (tp', T_rem, T_switch, T_total)."""
    t_cur = est_rem_time(pred, tp, groups, l_max, l_gen)
    t_best = math.inf
    tp_new = tp
    totals = []
    for cand in tp_list:
        merged = compute_merged(groups, n_gpus, cand)
        t_rem = est_rem_time(pred, cand, [merged], l_max, l_gen)
        t_sw = switch_cost_us(tp, cand, lengths, model, fixed_us, net_bytes_per_s, prefill, n_gpus)
        t_total = t_rem + t_sw
        totals.append((cand, t_rem, t_sw, t_total))
        if t_total < t_best:
            t_best = t_total
            tp_new = cand
    do_switch = tp_new != tp and t_cur > t_best
    return do_switch, tp_new, t_cur, t_best, totals
