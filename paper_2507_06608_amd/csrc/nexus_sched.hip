// C ABI of the phase-specific schedulers (declared in include/nexus.h): argument checks around nexus::Scheduler.
// Host code only.
#include <cmath>
#include <new>

#include "../../include/nexus.h"
#include "scheduler.hpp"
#include "status.hpp"

using namespace nexus;

struct nexus_sched {
    Scheduler impl;
    explicit nexus_sched(const nexus_sched_config &cfg) : impl(cfg) {}
};

extern "C" {

int nexus_sched_create(const nexus_sched_config *cfg, nexus_sched **out) {
    if (!cfg || !out) return fail(NEXUS_EINVAL, "null argument");
    if (cfg->prefill_policy != NEXUS_PREFILL_FCFS && cfg->prefill_policy != NEXUS_PREFILL_SPF) return fail(NEXUS_EINVAL, "unknown prefill policy %d", cfg->prefill_policy);
    if (cfg->token_budget < 1 || cfg->max_prefill_reqs < 0 || cfg->max_decode_reqs < 1) return fail(NEXUS_EINVAL, "token_budget and max_decode_reqs must be positive, max_prefill_reqs non-negative");
    if (cfg->page_size < 1 || cfg->n_pages < 1) return fail(NEXUS_EINVAL, "page_size and n_pages must be positive");
    if (cfg->reserved != 0 || (cfg->chunk_tail != 0 && cfg->chunk_tail != 1)) return fail(NEXUS_EINVAL, "reserved must be 0 and chunk_tail 0 or 1");
    if (!(cfg->gamma >= 0.0) || !std::isfinite(cfg->gamma)) return fail(NEXUS_EINVAL, "gamma must be finite and non-negative");
    if (cfg->page_order) {
        std::vector<char> seen(cfg->n_pages, 0);
        for (int32_t i = 0; i < cfg->n_pages; ++i) {
            const int32_t p = cfg->page_order[i];
            if (p < 0 || p >= cfg->n_pages || seen[p]) return fail(NEXUS_EINVAL, "page_order is not a permutation of 0..%d (entry %d = %d)", cfg->n_pages - 1, i, p);
            seen[p] = 1;
        }
    }
    nexus_sched *s = new (std::nothrow) nexus_sched(*cfg);
    if (!s) return fail(NEXUS_ENOMEM, "out of host memory");
    *out = s;
    return NEXUS_OK;
}

void nexus_sched_destroy(nexus_sched *s) { delete s; }

int nexus_sched_submit(nexus_sched *s, double arrival_s, int32_t prompt_len, int32_t output_len, int32_t *id_out) {
    if (!s) return fail(NEXUS_EINVAL, "null scheduler");
    if (!std::isfinite(arrival_s)) return fail(NEXUS_EINVAL, "arrival time must be finite");
    if (prompt_len < 1 || output_len < 1) return fail(NEXUS_EINVAL, "prompt_len %d and output_len %d must be at least 1", prompt_len, output_len);
    if (s->impl.lifetime_pages(prompt_len, output_len) > s->impl.total_pages())
        return fail(NEXUS_ESHAPE, "a request of %d + %d tokens needs more pages than the pool of %d", prompt_len, output_len, s->impl.total_pages());
    const int32_t id = s->impl.submit(arrival_s, prompt_len, output_len);
    if (id_out) *id_out = id;
    return NEXUS_OK;
}

int nexus_sched_next(nexus_sched *s, double now_s, nexus_sched_batch *out) {
    if (!s || !out) return fail(NEXUS_EINVAL, "null argument");
    if (!std::isfinite(now_s)) return fail(NEXUS_EINVAL, "time must be finite");
    if (s->impl.iteration_open() || s->impl.pending(NEXUS_PHASE_PREFILL) || s->impl.pending(NEXUS_PHASE_DECODE))
        return fail(NEXUS_ESTATE, "the previous iteration has not been committed");
    *out = nexus_sched_batch{};
    s->impl.next(now_s, out);
    return NEXUS_OK;
}

int nexus_sched_commit(nexus_sched *s, double end_s) {
    if (!s) return fail(NEXUS_EINVAL, "null scheduler");
    if (!s->impl.iteration_open()) return fail(NEXUS_ESTATE, "no iteration to commit");
    if (!(end_s >= s->impl.pending_now(NEXUS_PHASE_PREFILL))) return fail(NEXUS_EINVAL, "iteration ends (%g) before it starts (%g)", end_s, s->impl.pending_now(NEXUS_PHASE_PREFILL));
    s->impl.commit(end_s);
    return NEXUS_OK;
}

int nexus_sched_next_phase(nexus_sched *s, int phase, double now_s, nexus_sched_batch *out) {
    if (!s || !out) return fail(NEXUS_EINVAL, "null argument");
    if (phase != NEXUS_PHASE_PREFILL && phase != NEXUS_PHASE_DECODE) return fail(NEXUS_EINVAL, "unknown phase %d", phase);
    if (!std::isfinite(now_s)) return fail(NEXUS_EINVAL, "time must be finite");
    if (s->impl.iteration_open()) return fail(NEXUS_ESTATE, "a coupled iteration is open");
    if (s->impl.pending(phase)) return fail(NEXUS_ESTATE, "the previous tick of this phase has not been committed");
    *out = nexus_sched_batch{};
    if (phase == NEXUS_PHASE_PREFILL) s->impl.next_prefill(now_s, out);
    else s->impl.next_decode(now_s, out);
    return NEXUS_OK;
}

int nexus_sched_commit_phase(nexus_sched *s, int phase, double end_s) {
    if (!s) return fail(NEXUS_EINVAL, "null scheduler");
    if (phase != NEXUS_PHASE_PREFILL && phase != NEXUS_PHASE_DECODE) return fail(NEXUS_EINVAL, "unknown phase %d", phase);
    if (s->impl.iteration_open()) return fail(NEXUS_ESTATE, "a coupled iteration is open");
    if (!s->impl.pending(phase)) return fail(NEXUS_ESTATE, "this phase has no tick to commit");
    if (!(end_s >= s->impl.pending_now(phase))) return fail(NEXUS_EINVAL, "tick ends (%g) before it starts (%g)", end_s, s->impl.pending_now(phase));
    if (phase == NEXUS_PHASE_PREFILL) s->impl.commit_prefill(end_s);
    else s->impl.commit_decode(end_s);
    return NEXUS_OK;
}

int nexus_sched_request(const nexus_sched *s, int32_t id, nexus_sched_request_info *out) {
    if (!s || !out) return fail(NEXUS_EINVAL, "null argument");
    if (id < 0 || (size_t)id >= s->impl.size()) return fail(NEXUS_EINVAL, "no request %d", id);
    const Scheduler::Req &r = s->impl.request(id);
    out->arrival_s = r.arrival, out->first_token_s = r.first_s, out->finish_s = r.finish_s;
    out->prompt_len = r.prompt, out->output_len = r.output, out->prefilled = r.prefilled, out->emitted = r.emitted;
    out->n_pages = (int32_t)r.pages.size();
    out->state = r.finished ? 3 : r.in_pool ? 2 : r.ready ? 1 : 0;
    return NEXUS_OK;
}

static void collect(const Scheduler &s, int kind, std::vector<double> &v) {
    if (kind == 1) {
        v = s.tbt();
        return;
    }
    for (size_t i = 0; i < s.size(); ++i) {
        const Scheduler::Req &r = s.request(i);
        if (kind == 0 && r.first_s >= 0) v.push_back(r.first_s - r.arrival);
        if (kind == 2 && r.finished) v.push_back((r.finish_s - r.arrival) / r.output);
    }
}

int nexus_sched_samples(const nexus_sched *s, int kind, double *out, int32_t cap, int32_t *n) {
    if (!s || !n || (cap > 0 && !out) || cap < 0) return fail(NEXUS_EINVAL, "bad argument");
    if (kind < 0 || kind > 2) return fail(NEXUS_EINVAL, "unknown sample kind %d", kind);
    std::vector<double> v;
    collect(s->impl, kind, v);
    *n = (int32_t)v.size();
    for (int32_t i = 0; i < cap && i < *n; ++i) out[i] = v[i];
    return NEXUS_OK;
}

int nexus_sched_summarize(const nexus_sched *s, nexus_sched_summary *out) {
    if (!s || !out) return fail(NEXUS_EINVAL, "null argument");
    std::vector<double> ttft, tbt, nl;
    collect(s->impl, 0, ttft), collect(s->impl, 1, tbt), collect(s->impl, 2, nl);
    *out = nexus_sched_summary{};
    out->n_submitted = (int32_t)s->impl.size(), out->n_first_token = (int32_t)ttft.size(), out->n_finished = (int32_t)nl.size();
    out->prefill_tokens = s->impl.prefill_tokens(), out->decode_tokens = s->impl.decode_tokens();
    out->ttft_mean = mean(ttft), out->ttft_p50 = percentile(ttft, 0.5), out->ttft_p95 = percentile(ttft, 0.95);
    out->ttft_p99 = percentile(ttft, 0.99), out->ttft_max = percentile(ttft, 1.0);
    out->tbt_mean = mean(tbt), out->tbt_p50 = percentile(tbt, 0.5), out->tbt_p95 = percentile(tbt, 0.95);
    out->tbt_p99 = percentile(tbt, 0.99), out->tbt_max = percentile(tbt, 1.0);
    out->norm_latency_mean = mean(nl), out->norm_latency_p95 = percentile(nl, 0.95);
    return NEXUS_OK;
}

}  // extern "C"
