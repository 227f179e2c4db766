// Host side of the partition controller (Sec. 4.1-4.2): the analytic latency model of a phase on a share of the
// GPU (Eq. 5-7), decode's bandwidth under contention with prefill (Eq. 8-9), the two constrained objectives with
// their switch on KV-cache usage (Sec. 4.1.2), the greedy search and the buffer zone (Alg. 1), and the fit of an
// operator's saturation curve to measured times.  Plain C++ on host memory; no GPU work.
//
// Shares are integers: `share` of `total` equal steps (the paper counts percent, total = 100; on this chip a step
// is one CU in each of the 8 XCDs, total = 32).
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <utility>
#include <vector>

#include "../../include/nexus.h"

namespace nexus {

class CostModel {
public:
    explicit CostModel(const nexus_cost_model &m) : m_(m) {
        for (int i = 0; i < m.n_prefill_ops; ++i) {
            const nexus_cost_op &o = m.prefill_ops[i];
            (o.kind == NEXUS_OP_ATTENTION ? bytes_p_attn_ : bytes_p_dense_) += o.bytes;
        }
        for (int i = 0; i < m.n_decode_ops; ++i)
            if (m.decode_ops[i].kind == NEXUS_OP_ATTENTION) bytes_d_attn_ += m.decode_ops[i].bytes;
    }

    // Eq. 7: inverse scaling up to the saturation share, a linear decay (or growth) of the saturated time beyond.
    double compute_time(const nexus_cost_op &o, double r) const {
        const double t_sat = o.flops / (o.r_sat * m_.peak_flops);
        return r <= o.r_sat ? o.flops / (r * m_.peak_flops) : t_sat * (1.0 + o.lambda * (r - o.r_sat));
    }

    // Eq. 5 on the prefill operators (memory term at peak bandwidth); also returns the part spent in attention.
    double prefill_time(double r_p, double *attention_part = nullptr) const {
        double total = 0.0, attn = 0.0;
        for (int i = 0; i < m_.n_prefill_ops; ++i) {
            const nexus_cost_op &o = m_.prefill_ops[i];
            const double t = std::fmax(compute_time(o, r_p), o.bytes / m_.peak_bytes_per_s);
            total += t;
            if (o.kind == NEXUS_OP_ATTENTION) attn += t;
        }
        if (attention_part) *attention_part = attn;
        return total;
    }

    // Bandwidth left to decode attention next to a prefill phase on the share r_p (none when r_p == 0): decode's
    // fraction of the traffic while prefill is in attention (probability P_attn, Eq. 8) and while it is not.
    double decode_bandwidth(double r_p) const {
        if (r_p <= 0.0 || bytes_d_attn_ <= 0.0) return m_.peak_bytes_per_s;
        double attn = 0.0;
        const double t_p = prefill_time(r_p, &attn);
        const double p_attn = attn / t_p;
        const double in_attn = bytes_d_attn_ / (bytes_d_attn_ + bytes_p_attn_);
        const double in_dense = bytes_d_attn_ / (bytes_d_attn_ + bytes_p_dense_);
        return (in_attn * p_attn + in_dense * (1.0 - p_attn)) * m_.peak_bytes_per_s;
    }

    // Eq. 6 with Eq. 9 for the attention operators.
    double decode_time(double r_d, double r_p) const {
        const double bw_attn = decode_bandwidth(r_p);
        double total = 0.0;
        for (int i = 0; i < m_.n_decode_ops; ++i) {
            const nexus_cost_op &o = m_.decode_ops[i];
            const double mem = o.bytes / (o.kind == NEXUS_OP_ATTENTION ? bw_attn : m_.peak_bytes_per_s);
            total += std::fmax(compute_time(o, r_d), mem);
        }
        return total;
    }

    // CostModel(phase, R) of Alg. 1; the other phase holds the remaining steps, and never less than one: Alg. 1
    // takes its reference latency from this function at R = total, where Eq. 8 would otherwise have no value.
    double phase_time(int phase, int share, int total) const {
        const double r = (double)share / total, rest = (double)std::max(total - share, 1) / total;
        return phase == NEXUS_PHASE_PREFILL ? prefill_time(r) : decode_time(r, rest);
    }

    // AdjustPartition of Alg. 1.  `share` is the target phase's; both phases keep at least one step.
    int adjust(int target, int cur_prefill_share, int total, double alpha, double beta, int *evals) const {
        const int other = target == NEXUS_PHASE_PREFILL ? NEXUS_PHASE_DECODE : NEXUS_PHASE_PREFILL;
        const double budget = (target == NEXUS_PHASE_PREFILL ? beta : alpha) * phase_time(other, total, total);
        int n = 1;
        auto other_ok = [&](int target_share) {
            ++n;
            return phase_time(other, total - target_share, total) <= budget;
        };
        int share = target == NEXUS_PHASE_PREFILL ? cur_prefill_share : total - cur_prefill_share;
        if (share < 1) share = 1;
        if (share > total - 1) share = total - 1;
        while (share > 1 && !other_ok(share)) --share;             // constraint satisfaction
        while (share < total - 1 && other_ok(share + 1)) ++share;  // target optimisation
        if (evals) *evals = n;
        return target == NEXUS_PHASE_PREFILL ? share : total - share;
    }

private:
    const nexus_cost_model &m_;
    double bytes_p_attn_ = 0.0, bytes_p_dense_ = 0.0, bytes_d_attn_ = 0.0;
};

// Fit of Eq. 7 to measured (share, seconds) points of one operator: every measured share is tried as the
// saturation point; below it the effective work is the mean of t r C, above it lambda is the least-squares slope
// of the time relative to the saturated time; the candidate with the smallest squared relative error wins (the
// larger saturation point on ties).
inline void fit_saturation_curve(int n, const double *shares, const double *seconds, double peak_flops, double *flops,
                                 double *r_sat, double *lambda) {
    std::vector<std::pair<double, double>> pts(n);
    for (int i = 0; i < n; ++i) pts[i] = {shares[i], seconds[i]};
    std::sort(pts.begin(), pts.end());
    double best_err = INFINITY;
    for (int k = 0; k < n; ++k) {
        const double rs = pts[k].first;
        double work = 0.0;
        int below = 0;
        for (int i = 0; i < n; ++i)
            if (pts[i].first <= rs) work += pts[i].second * pts[i].first * peak_flops, ++below;
        work /= below;
        const double t_sat = work / (rs * peak_flops);
        double num = 0.0, den = 0.0;
        for (int i = 0; i < n; ++i)
            if (pts[i].first > rs) {
                const double dr = pts[i].first - rs;
                num += (pts[i].second / t_sat - 1.0) * dr;
                den += dr * dr;
            }
        const double lam = den > 0.0 ? num / den : 0.0;
        double err = 0.0;
        for (int i = 0; i < n; ++i) {
            const double r = pts[i].first;
            const double t = r <= rs ? work / (r * peak_flops) : t_sat * (1.0 + lam * (r - rs));
            const double e = (t - pts[i].second) / pts[i].second;
            err += e * e;
        }
        if (err <= best_err) best_err = err, *flops = work, *r_sat = rs, *lambda = lam;
    }
}

}  // namespace nexus
