// Latency predictor and online switch decision (host only): see include/pat_switch.h.
//
// The predictor keeps, per TP degree, the profiled batch sizes in ascending order with their
// fitted lines.  Because a query at a fixed batch size is itself a line in T (a blend of two
// lines with a fixed weight), the remaining decode time over n steps with T growing by B per
// step is an arithmetic series and is evaluated in closed form, not step by step.
#include "../../include/pat_switch.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <map>
#include <new>
#include <vector>

namespace {

struct Line { double alpha, beta; };

// least-squares line through (t, y); a single point or no spread in t gives the mean
Line fit(const std::vector<double> &t, const std::vector<double> &y)
{
    const size_t n = t.size();
    double mt = 0.0, my = 0.0;
    for (size_t i = 0; i < n; ++i) { mt += t[i]; my += y[i]; }
    mt /= (double)n; my /= (double)n;
    double stt = 0.0, sty = 0.0;
    for (size_t i = 0; i < n; ++i) { stt += (t[i] - mt) * (t[i] - mt); sty += (t[i] - mt) * (y[i] - my); }
    if (n == 1 || stt == 0.0) return {my, 0.0};
    const double beta = sty / stt;
    return {my - beta * mt, beta};
}

// batch sizes of one TP degree, ascending, with a payload each
template <class V>
struct ByBatch {
    std::vector<int32_t> batch;
    std::vector<V> val;
    // the two neighbours of `b` and the weight of the upper one
    void bracket(int32_t b, size_t *lo, size_t *hi, double *w) const
    {
        if (b <= batch.front()) { *lo = *hi = 0; *w = 0.0; return; }
        if (b >= batch.back()) { *lo = *hi = batch.size() - 1; *w = 0.0; return; }
        const size_t u = (size_t)(std::lower_bound(batch.begin(), batch.end(), b) - batch.begin());   // first >= b
        if (batch[u] == b) { *lo = *hi = u; *w = 0.0; return; }
        *lo = u - 1; *hi = u;
        *w = (double)(b - batch[u - 1]) / (double)(batch[u] - batch[u - 1]);
    }
};

}  // namespace

struct pat_predictor {
    std::map<int32_t, ByBatch<Line>> tp;
};

namespace {

// l(B, T) = a + b T for a fixed batch size
bool blend(const pat_predictor *p, int32_t tp, int32_t batch, Line *out)
{
    const auto it = p->tp.find(tp);
    if (it == p->tp.end() || batch < 1) return false;
    size_t lo, hi; double w;
    it->second.bracket(batch, &lo, &hi, &w);
    const Line &l0 = it->second.val[lo], &l1 = it->second.val[hi];
    *out = {(1.0 - w) * l0.alpha + w * l1.alpha, (1.0 - w) * l0.beta + w * l1.beta};
    return true;
}

// sum_{k < n} l(B, T + k B)
bool remaining(const pat_predictor *p, int32_t tp, int32_t batch, double T, int64_t n, double *out)
{
    *out = 0.0;
    if (batch <= 0 || n <= 0) return true;
    Line l;
    if (!blend(p, tp, batch, &l)) return false;
    const double nn = (double)n;
    *out = nn * l.alpha + l.beta * (nn * T + (double)batch * nn * (nn - 1.0) * 0.5);
    return true;
}

using Curve = std::vector<std::pair<double, double>>;      // (length, latency), ascending length

double curve_at(const Curve &c, double len)
{
    if (c.size() == 1) return c[0].second;
    size_t i = 0;
    while (i + 2 < c.size() && len > c[i + 1].first) ++i;
    return c[i].second + (c[i + 1].second - c[i].second) * (len - c[i].first) / (c[i + 1].first - c[i].first);
}

}  // namespace

extern "C" {

int pat_predictor_fit(const pat_grid_row *rows, int32_t n_rows, pat_predictor **out)
{
    if (!rows || n_rows <= 0 || !out) return PAT_EINVAL;
    std::map<std::pair<int32_t, int32_t>, std::pair<std::vector<double>, std::vector<double>>> pts;
    for (int32_t i = 0; i < n_rows; ++i) {
        const pat_grid_row &r = rows[i];
        if (r.skipped != 0) continue;
        if (r.tp_degree < 1 || r.batch < 1 || !(r.mean_us == r.mean_us)) return PAT_EINVAL;
        auto &p = pts[{r.tp_degree, r.batch}];
        p.first.push_back((double)r.sum_context);
        p.second.push_back(r.mean_us);
    }
    if (pts.empty()) return PAT_EINVAL;
    pat_predictor *p = new (std::nothrow) pat_predictor;
    if (!p) return PAT_ENOMEM;
    for (const auto &kv : pts) {                           // map order: tp, then batch ascending
        ByBatch<Line> &bb = p->tp[kv.first.first];
        bb.batch.push_back(kv.first.second);
        bb.val.push_back(fit(kv.second.first, kv.second.second));
    }
    *out = p;
    return PAT_OK;
}

void pat_predictor_destroy(pat_predictor *p) { delete p; }

int pat_predictor_line(const pat_predictor *p, int32_t tp, int32_t batch, double *alpha, double *beta)
{
    if (!p || !alpha || !beta) return PAT_EINVAL;
    const auto it = p->tp.find(tp);
    if (it == p->tp.end()) return PAT_EINVAL;
    const auto &b = it->second.batch;
    const auto f = std::lower_bound(b.begin(), b.end(), batch);
    if (f == b.end() || *f != batch) return PAT_EINVAL;
    const Line &l = it->second.val[(size_t)(f - b.begin())];
    *alpha = l.alpha; *beta = l.beta;
    return PAT_OK;
}

int pat_predictor_query(const pat_predictor *p, int32_t tp, int32_t batch, double sum_context, double *latency_us)
{
    Line l;
    if (!p || !latency_us || !blend(p, tp, batch, &l)) return PAT_EINVAL;
    *latency_us = l.alpha + l.beta * sum_context;
    return PAT_OK;
}

double pat_kv_move_seconds(const int32_t *lengths, int32_t n, int32_t n_layers, int32_t hidden, int32_t bytes_per_elem,
                           int32_t tp_src, double net_bytes_per_s)
{
    double s = 0.0;
    for (int32_t i = 0; i < n; ++i)
        s += 2.0 * (double)n_layers * (double)lengths[i] * ((double)hidden / (double)tp_src) * (double)bytes_per_elem;
    return s / net_bytes_per_s;
}

double pat_rms_length(const int32_t *lengths, int32_t n)
{
    double s = 0.0;
    for (int32_t i = 0; i < n; ++i) s += (double)lengths[i] * (double)lengths[i];
    return std::sqrt(s / (double)n);
}

// Sampling plan of the offline profiler (Sec. 4.1): see the header for the ladder this library takes.
int pat_profile_plan(int32_t n_gpus, int64_t t_cap, int64_t l_max, pat_plan_point *points, int32_t *n_points)
{
    if (!n_points || n_gpus < 1 || t_cap < 8 || l_max < 8) return PAT_EINVAL;
    static const int32_t kBatches[10] = {1, 2, 4, 8, 16, 32, 64, 128, 192, 256};
    std::vector<int64_t> lens;
    for (int64_t base = 8; base <= l_max; base *= 2) {
        lens.push_back(base);
        const int64_t mid = base + base / 2;                 // 12 * 2^i: the second point of an octave
        if (mid < 512 && mid <= l_max) lens.push_back(mid);
    }
    std::vector<pat_plan_point> plan;
    for (int32_t tp = 1; tp <= 8 && tp <= n_gpus; tp *= 2)
        for (int32_t b : kBatches)
            for (int64_t L : lens)
                if ((int64_t)b * L <= t_cap) plan.push_back(pat_plan_point{tp, b, (int32_t)L, 0});
    const int32_t cap = *n_points;
    if (points && cap < (int32_t)plan.size()) { *n_points = (int32_t)plan.size(); return PAT_ENOMEM; }
    if (points) std::copy(plan.begin(), plan.end(), points);
    *n_points = (int32_t)plan.size();
    return PAT_OK;
}

int pat_switch_decide(const pat_predictor *p, const pat_switch_input *in, pat_switch_decision *out)
{
    if (!p || !in || !out || !in->tp_list || in->n_tp < 1 || in->n_gpus < 1 || in->n_groups < 1 || !in->group_batch ||
        !in->group_context || !in->fixed_us || in->n_lengths < 0 || (in->n_lengths > 0 && !in->lengths) ||
        in->n_prefill < 0 || (in->n_prefill > 0 && !in->prefill) || !(in->net_bytes_per_s > 0.0))
        return PAT_EINVAL;
    int cur = -1;
    for (int32_t j = 0; j < in->n_tp; ++j) {
        const int32_t c = in->tp_list[j];
        if (c < 1 || in->n_gpus % c) return PAT_EINVAL;
        if (c == in->tp) cur = j;
    }
    if (cur < 0) return PAT_EINVAL;
    const int64_t steps = std::max<int64_t>(0, (int64_t)in->l_max - (int64_t)in->l_gen);

    // remaining time as things are: the slowest DP group
    double t_cur = 0.0;
    int64_t sum_b = 0; double sum_t = 0.0;
    for (int32_t g = 0; g < in->n_groups; ++g) {
        if (in->group_batch[g] < 0) return PAT_EINVAL;
        double r;
        if (!remaining(p, in->tp, in->group_batch[g], in->group_context[g], steps, &r)) return PAT_EINVAL;
        t_cur = std::max(t_cur, r);
        sum_b += in->group_batch[g]; sum_t += in->group_context[g];
    }

    // prefill curves of the recomputation estimate.  Eq. (4) reads a profiled latency: a row with a negative
    // or NaN latency is the profiler's mark of a pair it did not measure and is no point of a curve; a
    // (tp, batch) left without points has no curve, a degree left without curves no recomputation estimate.
    std::map<int32_t, ByBatch<Curve>> pre;
    if (in->n_prefill > 0) {
        std::map<std::pair<int32_t, int32_t>, Curve> c;
        for (int32_t i = 0; i < in->n_prefill; ++i) {
            const pat_prefill_row &r = in->prefill[i];
            if (!(r.latency_us >= 0.0)) continue;
            if (r.tp_degree < 1 || r.batch < 1 || r.length < 1) return PAT_EINVAL;
            c[{r.tp_degree, r.batch}].push_back({(double)r.length, r.latency_us});
        }
        for (auto &kv : c) {
            std::sort(kv.second.begin(), kv.second.end());
            for (size_t i = 1; i < kv.second.size(); ++i)
                if (kv.second[i].first == kv.second[i - 1].first) return PAT_EINVAL;    // a length measured twice
            ByBatch<Curve> &bb = pre[kv.first.first];
            bb.batch.push_back(kv.first.second);
            bb.val.push_back(kv.second);
        }
    }
    const double rms = in->n_lengths > 0 ? pat_rms_length(in->lengths, in->n_lengths) : 0.0;

    std::vector<double> rem((size_t)in->n_tp), sw((size_t)in->n_tp), tot((size_t)in->n_tp);
    double t_best = std::numeric_limits<double>::infinity();
    int32_t tp_new = in->tp;
    for (int32_t j = 0; j < in->n_tp; ++j) {
        const int32_t c = in->tp_list[j];
        const int64_t dp = in->n_gpus / c;
        const int64_t mb = (sum_b + dp - 1) / dp;
        if (!remaining(p, c, (int32_t)mb, sum_t / (double)dp, steps, &rem[(size_t)j])) return PAT_EINVAL;
        double cost = 0.0;
        if (c != in->tp) {
            const double t_move = 1e6 * pat_kv_move_seconds(in->lengths, in->n_lengths, in->n_layers, in->hidden,
                                                            in->bytes_per_elem, in->tp, in->net_bytes_per_s);
            double t_recomp = std::numeric_limits<double>::infinity();
            const auto it = pre.find(c);
            if (it != pre.end() && in->n_lengths > 0) {
                const int32_t bg = (int32_t)((in->n_lengths + dp - 1) / dp);
                size_t lo, hi; double w;
                it->second.bracket(bg, &lo, &hi, &w);
                t_recomp = (1.0 - w) * curve_at(it->second.val[lo], rms) + w * curve_at(it->second.val[hi], rms);
            }
            cost = in->fixed_us[(size_t)cur * (size_t)in->n_tp + (size_t)j] + std::min(t_move, t_recomp);
        }
        sw[(size_t)j] = cost;
        tot[(size_t)j] = rem[(size_t)j] + cost;
        if (tot[(size_t)j] < t_best) { t_best = tot[(size_t)j]; tp_new = c; }
    }
    out->do_switch = (tp_new != in->tp && t_cur > t_best) ? 1 : 0;
    out->tp_new = tp_new;
    out->t_cur_us = t_cur;
    out->t_best_us = t_best;
    for (int32_t j = 0; j < in->n_tp; ++j) {
        if (out->t_rem_us) out->t_rem_us[j] = rem[(size_t)j];
        if (out->t_switch_us) out->t_switch_us[j] = sw[(size_t)j];
        if (out->t_total_us) out->t_total_us[j] = tot[(size_t)j];
    }
    return PAT_OK;
}

}  // extern "C"
