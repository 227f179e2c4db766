// Sanitizer driver of the library's host-only code (test infrastructure): the schedulers, the partition controller,
// the split-selection rule and the validation of a step's integer inputs, exercised through the C ABI on seeded random
// input, including the error paths.  tests/test_sanitizers_host.py builds it together with nexus_host.hip and
// nexus_sched.hip as plain C++ (g++ -fsanitize=address,undefined); exit status 0 means no report and the checks held.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/nexus.h"

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static uint64_t next_u64() {
    uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}
static double uniform() { return (double)(next_u64() >> 11) / 9007199254740992.0; }
static int randint(int lo, int hi) { return lo + (int)(next_u64() % (uint64_t)(hi - lo + 1)); }

#define CHECK(c)                                                           \
    do {                                                                   \
        if (!(c)) {                                                        \
            fprintf(stderr, "check failed: %s (line %d): %s\n", #c, __LINE__, nexus_last_error()); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static int scheduler_run(int policy, bool phases) {
    std::vector<int32_t> order(48);
    for (int i = 0; i < 48; ++i) order[i] = 47 - i;
    nexus_sched_config cfg{};
    cfg.prefill_policy = policy, cfg.token_budget = 24, cfg.max_prefill_reqs = 3, cfg.max_decode_reqs = 4;
    cfg.page_size = 4, cfg.n_pages = 48, cfg.chunk_tail = 1, cfg.gamma = 15.0, cfg.page_order = order.data();
    nexus_sched *s = nullptr;
    CHECK(nexus_sched_create(&cfg, &s) == NEXUS_OK);
    double t = 0;
    int submitted = 0;
    for (int i = 0; i < 40; ++i) {
        t += uniform() * 0.05;
        int32_t id = -1;
        CHECK(nexus_sched_submit(s, t, randint(1, 70), randint(1, 12), &id) == NEXUS_OK && id == submitted);
        ++submitted;
    }
    CHECK(nexus_sched_submit(s, 0.0, 1000, 1, nullptr) == NEXUS_ESHAPE);  // lifetime larger than the pool
    CHECK(nexus_sched_submit(s, 0.0, 0, 1, nullptr) == NEXUS_EINVAL);
    double now = 0;
    for (int it = 0; it < 4000; ++it) {
        nexus_sched_batch b{};
        if (!phases) {
            CHECK(nexus_sched_next(s, now, &b) == NEXUS_OK);
            CHECK(nexus_sched_next(s, now, &b) == NEXUS_ESTATE);  // not committed yet
            long tokens = 0;
            for (int r = 0; r < b.n_prefill; ++r) {               // touch everything the batch points at
                tokens += b.prefill_chunk[r];
                const int pages = (b.prefill_prefix[r] + b.prefill_chunk[r] + 3) / 4;
                for (int p = 0; p < pages; ++p) CHECK(b.prefill_page_table[r * b.prefill_max_pages + p] >= 0);
            }
            CHECK(tokens == b.prefill_tokens && tokens <= 24 && b.n_decode <= 4);
            for (int j = 0; j < b.n_decode; ++j) CHECK(b.decode_page_table[j * b.decode_max_pages + b.decode_ctx[j] / 4] >= 0);
            now += 0.05;
            CHECK(nexus_sched_commit(s, now) == NEXUS_OK);
        } else {
            const int phase = it & 1;
            CHECK(nexus_sched_next_phase(s, phase, now, &b) == NEXUS_OK);
            now += phase ? 0.004 : 0.03;
            if (phase ? b.n_decode : b.n_prefill) CHECK(nexus_sched_commit_phase(s, phase, now) == NEXUS_OK);
        }
        nexus_sched_summary sum{};
        CHECK(nexus_sched_summarize(s, &sum) == NEXUS_OK);
        if (sum.n_finished == submitted) break;
    }
    nexus_sched_summary sum{};
    CHECK(nexus_sched_summarize(s, &sum) == NEXUS_OK);
    CHECK(sum.n_finished == submitted && sum.ttft_mean > 0 && sum.tbt_p99 >= sum.tbt_p50);
    for (int kind = 0; kind < 3; ++kind) {
        int32_t n = 0;
        CHECK(nexus_sched_samples(s, kind, nullptr, 0, &n) == NEXUS_OK && n > 0);
        std::vector<double> v(n);
        CHECK(nexus_sched_samples(s, kind, v.data(), n, &n) == NEXUS_OK);
    }
    nexus_sched_request_info info{};
    CHECK(nexus_sched_request(s, submitted - 1, &info) == NEXUS_OK && info.state == 3);
    CHECK(nexus_sched_request(s, submitted + 5, &info) != NEXUS_OK);
    nexus_sched_destroy(s);
    return 0;
}

int main() {
    for (int policy = 0; policy < 2; ++policy)
        for (int phases = 0; phases < 2; ++phases)
            if (scheduler_run(policy, phases != 0)) return 1;
    {
        nexus_sched_config bad{};
        nexus_sched *s = nullptr;
        CHECK(nexus_sched_create(&bad, &s) == NEXUS_EINVAL && nexus_sched_create(nullptr, &s) == NEXUS_EINVAL);
        nexus_sched_destroy(nullptr);
    }

    // partition controller
    nexus_model_desc desc{4096, 32, 8, 128, 14336, 1, 16, 1e-5f, 5e5f};
    nexus_cost_op pre[5], dec[5];
    CHECK(nexus_cost_describe(&desc, 1, 512, 917760, 2048, 64, 147456, pre, dec) == NEXUS_OK);
    for (int i = 0; i < 5; ++i) {
        double shares[8], secs[8], f, r, l;
        for (int k = 0; k < 8; ++k) {
            shares[k] = (k + 1) / 8.0;
            const double rs = 0.25 + 0.1 * i;
            secs[k] = (pre[i].flops + 1) / 2.5e15 / (shares[k] < rs ? shares[k] : rs) * (shares[k] > rs ? 1 - 0.3 * (shares[k] - rs) : 1.0) * (1 + 0.02 * uniform());
        }
        CHECK(nexus_cost_fit(8, shares, secs, 2.5e15, &f, &r, &l) == NEXUS_OK && r > 0 && r <= 1);
        pre[i].flops = f, pre[i].r_sat = r, pre[i].lambda = l;
        dec[i].r_sat = 0.375, dec[i].lambda = -0.4;
    }
    CHECK(nexus_cost_fit(0, nullptr, nullptr, 1, nullptr, nullptr, nullptr) == NEXUS_EINVAL);
    nexus_cost_model model{2.5e15, 8e12, 5, 5, pre, dec};
    for (int total : {8, 32, 100})
        for (int share = 1; share <= total; ++share)
            for (int phase = 0; phase < 2; ++phase) {
                double sec = -1;
                CHECK(nexus_cost_latency(&model, phase, share, total, &sec) == NEXUS_OK && sec > 0 && std::isfinite(sec));
            }
    double sec;
    CHECK(nexus_cost_latency(&model, 0, 0, 8, &sec) == NEXUS_EINVAL && nexus_cost_latency(&model, 2, 1, 8, &sec) == NEXUS_EINVAL);
    for (int cur = 0; cur <= 32; ++cur)
        for (int target = 0; target < 2; ++target) {
            int32_t out = -1, ev = -1;
            CHECK(nexus_adjust_partition(&model, target, cur, 32, 1.3, 1.1, &out, &ev) == NEXUS_OK && out >= 1 && out <= 31 && ev >= 1);
            CHECK(nexus_partition_controller(&model, target ? 0.9 : 0.1, 0.7, cur, 32, 1.3, 1.1, 2, &out) == NEXUS_OK);
        }
    int32_t out;
    CHECK(nexus_adjust_partition(&model, 0, 40, 32, 1.3, 1.1, &out, nullptr) == NEXUS_EINVAL);
    nexus_cost_model empty{2.5e15, 8e12, 0, 0, nullptr, nullptr};
    CHECK(nexus_cost_latency(&empty, 0, 4, 8, &sec) == NEXUS_OK && sec == 0.0);

    // split selection on random curves
    for (int trial = 0; trial < 500; ++trial) {
        const int n = randint(1, 9);
        std::vector<float> tp(n), td(n), ts(n);
        for (int i = 0; i < n; ++i) tp[i] = (float)(1 + uniform()), td[i] = (float)(1 + uniform()), ts[i] = tp[i] > td[i] ? tp[i] : td[i];
        for (int policy = 0; policy < 3; ++policy) {
            const int pick = nexus_choose_split(n, tp.data(), td.data(), ts.data(), 1.f, 1.f, policy, 1.3f, 1.1f);
            CHECK(pick >= 0 && pick < n);
        }
    }
    CHECK(nexus_choose_split(0, nullptr, nullptr, nullptr, 1, 1, 0, 1, 1) == NEXUS_EINVAL);

    // validation of a step's integer inputs: exact-size arrays, good and bad
    {
        const int32_t cu[3] = {0, 5, 12}, prefix[2] = {6, 0}, ptp[2 * 3] = {7, 2, 5, 0, 8, -1};
        const int32_t ctx[3] = {0, 3, 4}, ptd[3 * 2] = {4, -1, 1, -1, 6, 3};
        CHECK(nexus_validate_batches(9, 4, 2, 12, cu, prefix, ptp, 3, 7, 11, 3, ctx, ptd, 2, 5) == NEXUS_OK);
        CHECK(nexus_validate_batches(9, 4, 0, 0, nullptr, nullptr, nullptr, 0, 0, 0, 3, ctx, ptd, 2, 5) == NEXUS_OK);
        CHECK(nexus_validate_batches(8, 4, 2, 12, cu, prefix, ptp, 3, 7, 11, 3, ctx, ptd, 2, 5) == NEXUS_EINVAL);   // page 8 of 8
        CHECK(nexus_validate_batches(9, 4, 2, 12, cu, prefix, ptp, 3, 7, 10, 3, ctx, ptd, 2, 5) == NEXUS_EINVAL);   // total length hint
        CHECK(nexus_validate_batches(9, 4, 2, 13, cu, prefix, ptp, 3, 7, 11, 3, ctx, ptd, 2, 5) == NEXUS_EINVAL);   // token count
        const int32_t clash[3 * 2] = {4, -1, 7, -1, 6, 3};  // decode request 1 appends into a page prefill request 0 reads
        CHECK(nexus_validate_batches(9, 4, 2, 12, cu, prefix, ptp, 3, 7, 11, 3, ctx, clash, 2, 5) == NEXUS_EINVAL);
        CHECK(nexus_validate_batches(9, 4, 2, 12, nullptr, prefix, ptp, 3, 7, 11, 0, nullptr, nullptr, 0, 0) == NEXUS_EINVAL);
    }
    puts("host sanitizer driver: ok");
    return 0;
}
