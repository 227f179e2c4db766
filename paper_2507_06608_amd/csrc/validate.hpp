// Host-side validation of the integer contents of a step's batches: chunk offsets, prefix / context lengths and
// page tables (the arrays the kernels otherwise trust).  Plain C++, no GPU.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/nexus.h"
#include "status.hpp"

namespace nexus {

struct BatchView {  // every pointer is HOST memory; a batch with zero requests is absent
    int32_t n_pages, page_size;
    int32_t n_prefill_reqs, n_prefill_tokens;
    const int32_t *cu_chunk, *prefix_len, *prefill_page_table;
    int32_t prefill_max_pages, max_chunk, max_total_len;
    int32_t n_decode_reqs;
    const int32_t *ctx_len, *decode_page_table;
    int32_t decode_max_pages, max_ctx;
};

// A request reads pages [0, ceil(len / page_size)) of its table row, len being the positions it holds after the step,
// and writes the pages of the positions it appends.  Checked: offsets form an exclusive prefix sum ending at
// n_tokens; lengths are non-negative and within the hints that size the launch grids; every page a request touches
// is inside the pool and inside its table row; a page written by one request is touched by no other request of the
// step (two writers, or a reader next to a writer, would race between workgroups and between the two streams).
inline int validate_batches(const BatchView &v) {
    const int ps = v.page_size;
    std::vector<int32_t> writer(v.n_pages, -1);  // request index (prefill first, then decode) writing the page
    auto req_name = [&](int idx, char *buf, size_t n) {
        if (idx < v.n_prefill_reqs) snprintf(buf, n, "prefill request %d", idx);
        else snprintf(buf, n, "decode request %d", idx - v.n_prefill_reqs);
    };
    auto check_pages = [&](int idx, const int32_t *row, int32_t width, int64_t len, int64_t first_written) -> int {
        char who[48];
        req_name(idx, who, sizeof(who));
        const int64_t need = (len + ps - 1) / ps;
        if (need > width) return fail(NEXUS_EINVAL, "%s holds %lld positions, its page-table row has %d entries", who, (long long)len, width);
        for (int64_t i = 0; i < need; ++i) {
            const int32_t pg = row[i];
            if (pg < 0 || pg >= v.n_pages) return fail(NEXUS_EINVAL, "%s: page-table entry %lld is %d, outside the pool of %d pages", who, (long long)i, pg, v.n_pages);
            if (i >= first_written / ps) {
                if (writer[pg] >= 0 && writer[pg] != idx) {
                    char other[48];
                    req_name(writer[pg], other, sizeof(other));
                    return fail(NEXUS_EINVAL, "page %d is written by %s and by %s", pg, other, who);
                }
                writer[pg] = idx;
            }
        }
        return NEXUS_OK;
    };
    if (v.n_prefill_reqs > 0) {
        if (v.cu_chunk[0] != 0) return fail(NEXUS_EINVAL, "cu_chunk[0] is %d, must be 0", v.cu_chunk[0]);
        if (v.cu_chunk[v.n_prefill_reqs] != v.n_prefill_tokens)
            return fail(NEXUS_EINVAL, "cu_chunk ends at %d, n_tokens is %d", v.cu_chunk[v.n_prefill_reqs], v.n_prefill_tokens);
    }
    for (int r = 0; r < v.n_prefill_reqs; ++r) {
        const int64_t n = (int64_t)v.cu_chunk[r + 1] - v.cu_chunk[r], pre = v.prefix_len[r];
        if (n < 0) return fail(NEXUS_EINVAL, "cu_chunk decreases at prefill request %d", r);
        if (n > v.max_chunk) return fail(NEXUS_EINVAL, "prefill request %d: chunk of %lld tokens exceeds max_chunk %d", r, (long long)n, v.max_chunk);
        if (pre < 0) return fail(NEXUS_EINVAL, "prefill request %d: negative prefix_len %lld", r, (long long)pre);
        if (pre + n > v.max_total_len) return fail(NEXUS_EINVAL, "prefill request %d: %lld positions exceed max_total_len %d", r, (long long)(pre + n), v.max_total_len);
        if (n == 0) continue;
        const int rc = check_pages(r, v.prefill_page_table + (size_t)r * v.prefill_max_pages, v.prefill_max_pages, pre + n, pre);
        if (rc) return rc;
    }
    for (int j = 0; j < v.n_decode_reqs; ++j) {
        const int64_t c = v.ctx_len[j];
        if (c < 0) return fail(NEXUS_EINVAL, "decode request %d: negative ctx_len %lld", j, (long long)c);
        if (c + 1 > v.max_ctx) return fail(NEXUS_EINVAL, "decode request %d: %lld positions exceed max_ctx %d", j, (long long)(c + 1), v.max_ctx);
        const int rc = check_pages(v.n_prefill_reqs + j, v.decode_page_table + (size_t)j * v.decode_max_pages, v.decode_max_pages, c + 1, c);
        if (rc) return rc;
    }
    // a page one request writes must not be read by another either
    auto check_readers = [&](int idx, const int32_t *row, int64_t first_written) -> int {
        for (int64_t i = 0; i < first_written / ps; ++i) {
            const int32_t pg = row[i];
            if (writer[pg] >= 0 && writer[pg] != idx) {
                char who[48], other[48];
                req_name(idx, who, sizeof(who)), req_name(writer[pg], other, sizeof(other));
                return fail(NEXUS_EINVAL, "page %d is read by %s while %s writes it", pg, who, other);
            }
        }
        return NEXUS_OK;
    };
    for (int r = 0; r < v.n_prefill_reqs; ++r) {
        if (v.cu_chunk[r + 1] == v.cu_chunk[r]) continue;
        const int rc = check_readers(r, v.prefill_page_table + (size_t)r * v.prefill_max_pages, v.prefix_len[r]);
        if (rc) return rc;
    }
    for (int j = 0; j < v.n_decode_reqs; ++j) {
        const int rc = check_readers(v.n_prefill_reqs + j, v.decode_page_table + (size_t)j * v.decode_max_pages, v.ctx_len[j]);
        if (rc) return rc;
    }
    return NEXUS_OK;
}

}  // namespace nexus
