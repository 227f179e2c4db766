// Host-only part of the C ABI declared in include/nexus.h: the split-selection rule on measured curves, the
// partition controller (cost model, greedy search, buffer zone, curve fit) and the host-side validation of a step's
// integer inputs.  No GPU call and no HIP header: this file and nexus_sched.hip also build with a plain C++ compiler
// (the sanitizer build of the CPU tests does that).
#include <algorithm>
#include <cmath>
#include <cstdlib>

#include "../../include/nexus.h"
#include "cost_model.hpp"
#include "status.hpp"
#include "validate.hpp"

using namespace nexus;

#define NX_TRY(expr)             \
    do {                         \
        int s_ = (expr);         \
        if (s_ != NEXUS_OK) return s_; \
    } while (0)

extern "C" {

const char *nexus_last_error(void) { return g_err; }

// The selection rule; kept free of HIP so that the host tests can drive it with synthetic curves.
int nexus_choose_split(int n, const float *t_p, const float *t_d, const float *t_step, float t_p_all, float t_d_all, int policy, float alpha,
                       float beta) {
    if (n <= 0 || !t_p || !t_d || !t_step) return fail(NEXUS_EINVAL, "bad curve arguments");
    if (policy < 0 || policy > 2) return fail(NEXUS_EINVAL, "unknown policy %d", policy);
    int best = -1;
    if (policy == NEXUS_POLICY_MIN_STEP) {
        for (int i = 0; i < n; ++i)
            if (best < 0 || t_step[i] < t_step[best]) best = i;
        return best;
    }
    const bool pp = policy == NEXUS_POLICY_PREFILL_PRIORITIZED;
    const float *obj = pp ? t_p : t_d, *con = pp ? t_d : t_p;
    const double bound = pp ? (double)beta * t_d_all : (double)alpha * t_p_all;
    for (int i = 0; i < n; ++i)
        if ((double)con[i] <= bound && (best < 0 || obj[i] < obj[best])) best = i;
    if (best < 0)  // nothing meets the slack: take the candidate that violates it least
        for (int i = 0; i < n; ++i)
            if (best < 0 || con[i] < con[best]) best = i;
    return best;
}

// ---------------------------------------------------------------------------------------------- partition controller
static int check_cost_model(const nexus_cost_model *m) {
    if (!m || (m->n_prefill_ops > 0 && !m->prefill_ops) || (m->n_decode_ops > 0 && !m->decode_ops)) return fail(NEXUS_EINVAL, "null cost model");
    if (m->n_prefill_ops < 0 || m->n_decode_ops < 0) return fail(NEXUS_EINVAL, "negative operator count");
    if (!(m->peak_flops > 0.0) || !(m->peak_bytes_per_s > 0.0)) return fail(NEXUS_EINVAL, "peak throughput and bandwidth must be positive");
    for (int p = 0; p < 2; ++p) {
        const nexus_cost_op *ops = p ? m->decode_ops : m->prefill_ops;
        for (int i = 0; i < (p ? m->n_decode_ops : m->n_prefill_ops); ++i) {
            if (!(ops[i].r_sat > 0.0) || ops[i].r_sat > 1.0) return fail(NEXUS_EINVAL, "operator %d: r_sat %g outside (0, 1]", i, ops[i].r_sat);
            if (ops[i].flops < 0.0 || ops[i].bytes < 0.0) return fail(NEXUS_EINVAL, "operator %d: negative work", i);
            if (ops[i].kind != NEXUS_OP_DENSE && ops[i].kind != NEXUS_OP_ATTENTION) return fail(NEXUS_EINVAL, "operator %d: bad kind", i);
        }
    }
    return NEXUS_OK;
}

int nexus_cost_latency(const nexus_cost_model *model, int phase, int share, int total, double *seconds) {
    NX_TRY(check_cost_model(model));
    if (!seconds) return fail(NEXUS_EINVAL, "null output");
    if (phase != NEXUS_PHASE_PREFILL && phase != NEXUS_PHASE_DECODE) return fail(NEXUS_EINVAL, "bad phase %d", phase);
    if (total < 1 || share < 1 || share > total) return fail(NEXUS_EINVAL, "share %d of %d", share, total);
    *seconds = CostModel(*model).phase_time(phase, share, total);
    return NEXUS_OK;
}

int nexus_adjust_partition(const nexus_cost_model *model, int target_phase, int cur_prefill_share, int total, double alpha,
                           double beta, int32_t *new_prefill_share, int32_t *evaluations) {
    NX_TRY(check_cost_model(model));
    if (!new_prefill_share) return fail(NEXUS_EINVAL, "null output");
    if (target_phase != NEXUS_PHASE_PREFILL && target_phase != NEXUS_PHASE_DECODE) return fail(NEXUS_EINVAL, "bad phase %d", target_phase);
    if (total < 2 || cur_prefill_share < 0 || cur_prefill_share > total) return fail(NEXUS_EINVAL, "prefill share %d of %d", cur_prefill_share, total);
    if (!(alpha >= 1.0) || !(beta >= 1.0)) return fail(NEXUS_EINVAL, "slack factors must be >= 1");
    int n = 0;
    *new_prefill_share = CostModel(*model).adjust(target_phase, cur_prefill_share, total, alpha, beta, &n);
    if (evaluations) *evaluations = n;
    return NEXUS_OK;
}

int nexus_partition_controller(const nexus_cost_model *model, double kv_usage, double kv_switch, int cur_prefill_share,
                               int total, double alpha, double beta, int delta, int32_t *new_prefill_share) {
    if (delta < 0) return fail(NEXUS_EINVAL, "negative buffer zone");
    int32_t proposed = 0;
    const int target = kv_usage > kv_switch ? NEXUS_PHASE_DECODE : NEXUS_PHASE_PREFILL;
    NX_TRY(nexus_adjust_partition(model, target, cur_prefill_share, total, alpha, beta, &proposed, nullptr));
    *new_prefill_share = std::abs(proposed - cur_prefill_share) < delta ? cur_prefill_share : proposed;
    return NEXUS_OK;
}

int nexus_cost_fit(int n, const double *shares, const double *seconds, double peak_flops, double *flops, double *r_sat, double *lambda) {
    if (n < 1 || !shares || !seconds || !flops || !r_sat || !lambda) return fail(NEXUS_EINVAL, "bad argument");
    if (!(peak_flops > 0.0)) return fail(NEXUS_EINVAL, "peak throughput must be positive");
    for (int i = 0; i < n; ++i)
        if (!(shares[i] > 0.0) || shares[i] > 1.0 || !(seconds[i] > 0.0)) return fail(NEXUS_EINVAL, "point %d: share %g, %g s", i, shares[i], seconds[i]);
    fit_saturation_curve(n, shares, seconds, peak_flops, flops, r_sat, lambda);
    return NEXUS_OK;
}

int nexus_cost_describe(const nexus_model_desc *d, int layers, double prefill_tokens, double prefill_pairs, double prefill_kv_tokens,
                        double decode_reqs, double decode_kv_tokens, nexus_cost_op *prefill_ops, nexus_cost_op *decode_ops) {
    if (!d || !prefill_ops || !decode_ops || layers < 1) return fail(NEXUS_EINVAL, "bad argument");
    const double q_dim = (double)d->n_q_heads * d->head_dim, kv_dim = (double)d->n_kv_heads * d->head_dim;
    const double out_rows[5] = {q_dim + 2 * kv_dim, 0, (double)d->hidden, 2.0 * d->ffn, (double)d->hidden};
    const double in_cols[5] = {(double)d->hidden, 0, q_dim, (double)d->hidden, (double)d->ffn};
    const double kv_token_bytes = 2.0 * kv_dim * 2.0;  // K and V, two bytes each
    for (int i = 0; i < 5; ++i) {
        nexus_cost_op p{}, q{};
        p.r_sat = q.r_sat = 1.0;
        if (i == 1) {
            p.kind = q.kind = NEXUS_OP_ATTENTION;
            p.flops = 4.0 * d->head_dim * d->n_q_heads * prefill_pairs;  // QK^T and PV, two flops per multiply-add
            p.bytes = prefill_kv_tokens * kv_token_bytes;
            q.flops = 4.0 * d->head_dim * d->n_q_heads * decode_kv_tokens;
            q.bytes = decode_kv_tokens * kv_token_bytes;
        } else {
            const double weights = out_rows[i] * in_cols[i];
            p.kind = q.kind = NEXUS_OP_DENSE;
            p.flops = 2.0 * prefill_tokens * weights, p.bytes = 2.0 * weights;
            q.flops = 2.0 * decode_reqs * weights, q.bytes = 2.0 * weights;
        }
        p.flops *= layers, p.bytes *= layers, q.flops *= layers, q.bytes *= layers;
        prefill_ops[i] = p, decode_ops[i] = q;
    }
    return NEXUS_OK;
}

int nexus_validate_batches(int32_t n_pages, int32_t page_size, int32_t n_prefill_reqs, int32_t n_prefill_tokens,
                           const int32_t *cu_chunk, const int32_t *prefix_len, const int32_t *prefill_page_table,
                           int32_t prefill_max_pages, int32_t max_chunk, int32_t max_total_len, int32_t n_decode_reqs,
                           const int32_t *ctx_len, const int32_t *decode_page_table, int32_t decode_max_pages, int32_t max_ctx) {
    if (n_pages <= 0 || page_size <= 0) return fail(NEXUS_EINVAL, "n_pages and page_size must be positive");
    if (n_prefill_reqs < 0 || n_decode_reqs < 0) return fail(NEXUS_EINVAL, "negative request count");
    if (n_prefill_reqs > 0 && (!cu_chunk || !prefix_len || !prefill_page_table || prefill_max_pages <= 0)) return fail(NEXUS_EINVAL, "null array in the prefill batch");
    if (n_decode_reqs > 0 && (!ctx_len || !decode_page_table || decode_max_pages <= 0)) return fail(NEXUS_EINVAL, "null array in the decode batch");
    BatchView v{n_pages, page_size, n_prefill_reqs, n_prefill_tokens, cu_chunk, prefix_len, prefill_page_table, prefill_max_pages,
                max_chunk, max_total_len, n_decode_reqs, ctx_len, decode_page_table, decode_max_pages, max_ctx};
    return validate_batches(v);
}

}  // extern "C"
