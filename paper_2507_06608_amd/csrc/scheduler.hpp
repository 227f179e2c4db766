// Host side of the phase-specific schedulers (Sec. 4.3): Shortest Prompt First with the age term (Eq. 10, Alg. 2)
// or FCFS for the prefill queue, FCFS for the decode pool, and the per-iteration bookkeeping around them -- chunk
// progress, page allocation from a free list, token times -- that turns a stream of requests into the batch
// descriptors the step calls take.  Plain C++ on host memory; no GPU work.
//
// One tick of a phase is next_<phase>(now) -> the caller runs that phase's step -> commit_<phase>(end); the coupled
// iteration next(now) / commit(end) is one tick of each.  A request emits its first token when its last prompt
// chunk commits, then waits for a place in the decode pool (first prefilled, first served) and emits one token
// per committed decode tick until it has produced output_len tokens.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/nexus.h"

namespace nexus {

class Scheduler {
public:
    struct Req {
        double arrival;
        int32_t prompt, output;
        int32_t prefilled = 0, emitted = 0, reserved = 0;
        bool admitted = false, in_pool = false, ready = false, finished = false;
        double ready_s = 0, first_s = -1, last_s = -1, finish_s = -1;
        std::vector<int32_t> pages;
    };

    explicit Scheduler(const nexus_sched_config &cfg) : cfg_(cfg) {
        free_.resize(cfg.n_pages);
        for (int32_t i = 0; i < cfg.n_pages; ++i)  // back() is handed out first
            free_[cfg.n_pages - 1 - i] = cfg.page_order ? cfg.page_order[i] : i;
        cfg_.page_order = nullptr;
    }

    int32_t pages_for(int64_t tokens) const { return (int32_t)((tokens + cfg_.page_size - 1) / cfg_.page_size); }
    int32_t lifetime_pages(int32_t prompt, int32_t output) const { return pages_for((int64_t)prompt + output - 1); }
    int32_t total_pages() const { return cfg_.n_pages; }
    size_t size() const { return reqs_.size(); }
    const Req &request(size_t i) const { return reqs_[i]; }
    int64_t prefill_tokens() const { return prefill_tokens_; }
    int64_t decode_tokens() const { return decode_tokens_; }
    const std::vector<double> &tbt() const { return tbt_; }

    int32_t submit(double arrival, int32_t prompt, int32_t output) {
        Req r;
        r.arrival = arrival, r.prompt = prompt, r.output = output;
        reqs_.push_back(std::move(r));
        waiting_.push_back((int32_t)reqs_.size() - 1);
        return (int32_t)reqs_.size() - 1;
    }

    // The two phases tick independently (Sec. 5: separate coroutines, each with its own scheduler).  An empty
    // batch is not pending: there is nothing to commit.
    bool pending(int phase) const { return phase == NEXUS_PHASE_PREFILL ? prefill_pending_ : decode_pending_; }
    double pending_now(int phase) const { return phase == NEXUS_PHASE_PREFILL ? prefill_now_ : decode_now_; }

    void next_prefill(double now, nexus_sched_batch *out) {
        prefill_now_ = now;
        // -- prefill queue: visible, not fully prefilled, in policy order (Alg. 2: score, sort)
        std::vector<Key> order;
        for (int32_t id : waiting_) {
            const Req &r = reqs_[id];
            if (r.arrival > now) continue;
            const double score = cfg_.prefill_policy == NEXUS_PREFILL_SPF
                                     ? (double)(r.prompt - r.prefilled) - cfg_.gamma * (now - r.arrival)
                                     : 0.0;
            order.push_back({score, r.arrival, id});
        }
        std::sort(order.begin(), order.end());
        // -- admission: a request that cannot reserve its lifetime's pages holds back every new request behind it
        std::vector<int32_t> admitted;
        bool blocked = false;
        for (const Key &k : order) {
            Req &r = reqs_[k.id];
            if (!r.admitted) {
                const int32_t need = lifetime_pages(r.prompt, r.output);
                if (blocked || reserved_total_ + need > cfg_.n_pages) {
                    blocked = true;
                    continue;
                }
                r.admitted = true, r.reserved = need;
                reserved_total_ += need;
            }
            admitted.push_back(k.id);
        }
        // -- Alg. 2, the filling loop (with the chunked-prefill tail)
        p_req_.clear(), p_prefix_.clear(), p_chunk_.clear();
        int32_t total = 0;
        for (int32_t id : admitted) {
            if (cfg_.max_prefill_reqs > 0 && (int32_t)p_req_.size() == cfg_.max_prefill_reqs) break;
            const Req &r = reqs_[id];
            const int32_t remaining = r.prompt - r.prefilled;
            int32_t take = 0;
            if (total + remaining <= cfg_.token_budget) take = remaining;
            else if (cfg_.chunk_tail) take = cfg_.token_budget - total;
            if (take > 0) p_req_.push_back(id), p_prefix_.push_back(r.prefilled), p_chunk_.push_back(take), total += take;
            if (take < remaining) break;
        }
        for (size_t i = 0; i < p_req_.size(); ++i) grow(reqs_[p_req_[i]], (int64_t)p_prefix_[i] + p_chunk_[i]);
        prefill_pending_ = !p_req_.empty();
        describe_prefill(out, total);
    }

    void next_decode(double now, nexus_sched_batch *out) {
        decode_now_ = now;
        // -- decode pool: first prefilled, first served
        std::vector<Key> ready;
        for (int32_t id : ready_) ready.push_back({reqs_[id].ready_s, reqs_[id].arrival, id});
        std::sort(ready.begin(), ready.end());
        ready_.clear();
        for (const Key &k : ready) {
            if ((int32_t)pool_.size() < cfg_.max_decode_reqs) reqs_[k.id].in_pool = true, pool_.push_back(k.id);
            else ready_.push_back(k.id);
        }
        d_req_.clear(), d_ctx_.clear();
        for (int32_t id : pool_) {
            Req &r = reqs_[id];
            const int32_t ctx = r.prompt + r.emitted - 1;
            grow(r, (int64_t)ctx + 1);
            d_req_.push_back(id), d_ctx_.push_back(ctx);
        }
        decode_pending_ = !d_req_.empty();
        describe_decode(out);
    }

    // Token times and progress of a completed tick; finished requests release their pages.
    void commit_decode(double end) {
        std::vector<int32_t> still;
        for (int32_t id : pool_) {
            Req &r = reqs_[id];
            ++r.emitted, ++decode_tokens_;
            tbt_.push_back(end - r.last_s);
            r.last_s = end;
            if (r.emitted == r.output) r.in_pool = false, finish(r, end);
            else still.push_back(id);
        }
        pool_.swap(still);
        d_req_.clear(), d_ctx_.clear();
        decode_pending_ = false;
    }

    void commit_prefill(double end) {
        for (size_t i = 0; i < p_req_.size(); ++i) {
            Req &r = reqs_[p_req_[i]];
            r.prefilled += p_chunk_[i], prefill_tokens_ += p_chunk_[i];
            if (r.prefilled == r.prompt) {
                r.emitted = 1, r.first_s = r.last_s = end;
                waiting_.erase(std::find(waiting_.begin(), waiting_.end(), p_req_[i]));
                if (r.output == 1) finish(r, end);
                else r.ready = true, r.ready_s = end, ready_.push_back(p_req_[i]);
            }
        }
        p_req_.clear(), p_prefix_.clear(), p_chunk_.clear();
        prefill_pending_ = false;
    }

    // The coupled iteration: one tick of each phase, started together and committed together.
    bool iteration_open() const { return iteration_open_; }
    void next(double now, nexus_sched_batch *out) {
        next_prefill(now, out);
        next_decode(now, out);
        iteration_open_ = true;
    }
    void commit(double end) {
        if (decode_pending_) commit_decode(end);
        if (prefill_pending_) commit_prefill(end);
        iteration_open_ = false;
    }

private:
    struct Key {
        double primary, arrival;
        int32_t id;
        bool operator<(const Key &o) const {
            if (primary != o.primary) return primary < o.primary;
            if (arrival != o.arrival) return arrival < o.arrival;
            return id < o.id;
        }
    };

    void grow(Req &r, int64_t tokens) {
        while ((int32_t)r.pages.size() < pages_for(tokens)) r.pages.push_back(free_.back()), free_.pop_back();
    }
    void finish(Req &r, double end) {
        r.finished = true, r.finish_s = end;
        for (size_t i = r.pages.size(); i-- > 0;) free_.push_back(r.pages[i]);
        r.pages.clear();
        reserved_total_ -= r.reserved, r.reserved = 0;
    }
    static void table(const std::vector<Req> &reqs, const std::vector<int32_t> &ids, std::vector<int32_t> &t, int32_t *width) {
        size_t w = 1;
        for (int32_t id : ids) w = std::max(w, reqs[id].pages.size());
        t.assign(ids.size() * w, -1);  // entries past a request's own pages must never be dereferenced
        for (size_t i = 0; i < ids.size(); ++i) std::copy(reqs[ids[i]].pages.begin(), reqs[ids[i]].pages.end(), t.begin() + i * w);
        *width = (int32_t)w;
    }
    void describe_prefill(nexus_sched_batch *b, int32_t total) {
        p_cu_.assign(p_req_.size() + 1, 0);
        int32_t max_chunk = 0, max_total = 0;
        for (size_t i = 0; i < p_req_.size(); ++i) {
            p_cu_[i + 1] = p_cu_[i] + p_chunk_[i];
            max_chunk = std::max(max_chunk, p_chunk_[i]);
            max_total = std::max(max_total, p_prefix_[i] + p_chunk_[i]);
        }
        table(reqs_, p_req_, p_table_, &b->prefill_max_pages);
        b->n_prefill = (int32_t)p_req_.size(), b->prefill_tokens = total;
        b->prefill_req = p_req_.data(), b->prefill_prefix = p_prefix_.data(), b->prefill_chunk = p_chunk_.data();
        b->prefill_cu_chunk = p_cu_.data(), b->prefill_page_table = p_table_.data();
        b->prefill_max_chunk = max_chunk, b->prefill_max_total_len = max_total;
        b->kv_used_pages = cfg_.n_pages - (int32_t)free_.size(), b->kv_total_pages = cfg_.n_pages;
    }
    void describe_decode(nexus_sched_batch *b) {
        int32_t max_ctx = 0;
        for (int32_t c : d_ctx_) max_ctx = std::max(max_ctx, c);
        table(reqs_, d_req_, d_table_, &b->decode_max_pages);
        b->n_decode = (int32_t)d_req_.size();
        b->decode_req = d_req_.data(), b->decode_ctx = d_ctx_.data(), b->decode_page_table = d_table_.data();
        b->decode_max_ctx = max_ctx;
        b->kv_used_pages = cfg_.n_pages - (int32_t)free_.size(), b->kv_total_pages = cfg_.n_pages;
    }

    nexus_sched_config cfg_;
    std::vector<Req> reqs_;
    std::vector<int32_t> waiting_, ready_, pool_, free_;
    std::vector<int32_t> p_req_, p_prefix_, p_chunk_, p_cu_, p_table_, d_req_, d_ctx_, d_table_;
    std::vector<double> tbt_;
    int64_t reserved_total_ = 0, prefill_tokens_ = 0, decode_tokens_ = 0;
    double prefill_now_ = 0, decode_now_ = 0;
    bool prefill_pending_ = false, decode_pending_ = false, iteration_open_ = false;
};

// Nearest-rank percentile (the smallest sample with at least q of the samples at or below it); 0 for no samples.
inline double percentile(std::vector<double> v, double q) {
    if (v.empty()) return 0.0;
    std::sort(v.begin(), v.end());
    size_t k = (size_t)std::ceil(q * (double)v.size());
    if (k < 1) k = 1;
    return v[std::min(k, v.size()) - 1];
}
inline double mean(const std::vector<double> &v) {
    double s = 0;
    for (double x : v) s += x;
    return v.empty() ? 0.0 : s / (double)v.size();
}

}  // namespace nexus
