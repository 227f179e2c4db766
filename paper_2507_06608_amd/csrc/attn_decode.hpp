// Paged grouped-query decode attention (Sec. 2.3: one query token per request against all of its cached keys; a
// memory-bound sweep over the KV cache), split over the context, plus the merge of the split results.
//
// Work item = (request, kv head, span of kSpan keys), one wavefront each, independent of every other work item.
// The span boundaries depend on the context length only, so the reduction order is the same on any CU share.
// The wavefront serves all G query heads of its kv head at once, so every K/V byte is fetched once per kv head.
// K and V pages are read straight from global memory into MFMA operand registers: the private page layouts make
// each load instruction cover contiguous runs of memory with 16 bytes per lane, and no LDS is needed because
// nothing is shared between wavefronts.  The products run on v_mfma_f32_16x16x32_bf16 with the G query heads
// padded to the 16 columns of the tile; on this memory-bound sweep the matrix unit is otherwise idle, while the
// same work on the vector ALUs would cost about G+1 instructions per KV element and bind before HBM does once
// the phase only owns a fraction of the CUs.  As in the prefill kernel the transposed orientation
// (S^T = K Q^T, O^T = V^T P^T) keeps softmax statistics per lane and lets the S^T accumulators serve directly as
// the P^T operand.  The loop is kept lean on purpose (no per-load predicates, raw v_exp_f32): with a dozen VALU
// instructions per key the sweep would be instruction-bound, not memory-bound.
#pragma once
#include "common.hpp"

namespace nexus {

constexpr int kSpan = 256;  // keys per work item (16 pages)
constexpr int kDecWaves = 1;  // work items (wavefronts) per workgroup

struct AttnDecodeArgs {
    const bf16_t *q;  // row-major [B][Hq*hd], rotated
    const int32_t *ctx_len, *page_table;
    int n_reqs, max_pages, max_spans;
    const bf16_t *k_pool, *v_pool;
    int n_pages, Hq, Hkv;
    float scale_log2e;
    f16_t *part_o;   // [B][Hkv][max_spans][G][hd]: each span's output normalised by its own sum, half
    float *part_ml;  // [B][Hkv][max_spans][G][2]  (running max in the log2 domain, sum)
    f16_t *out;      // merge output: half, P32 [B rows][Hq*hd]
    // Decode requests riding in a chunked-prefill batch (the fused single-batch step): their queries sit in the
    // prefill layout -- P32, every request on a 32-row boundary, request j of the decode part in the row tile that
    // follows the tiles of the n_lead leading requests -- and their outputs go to rows out_row0 + j.  lead_cu is
    // null for the plain decode phase (q row-major [B][Hq*hd], output row j).
    const int32_t *lead_cu;  // cu_chunk of the batch the requests ride in
    int n_lead, out_row0;
};

template <int HD, int G>
__global__ __launch_bounds__(kDecWaves * 64, 2) void attn_decode_kernel(AttnDecodeArgs a) {
    constexpr int KK = HD / 32;   // k-steps of QK^T
    constexpr int RT = HD / 16;   // 16-row tiles of O^T
    constexpr int BLK = kPage * HD;  // elements per (page, kv head) block
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // Work items are numbered span-major: workgroups are dealt to the 8 XCDs round-robin, and with the span index
    // running fastest each XCD would always serve the same span positions -- the first spans, which every
    // request has, on some XCDs and the rarely present last spans on others (measured: 1.4x the time of a
    // balanced launch on a third of the chip).  Span-major, each span's (request, kv head) items spread evenly.
    const int wi = blockIdx.x * kDecWaves + w;
    const int per_span = a.n_reqs * a.Hkv;
    const int span = wi / per_span;
    if (span >= a.max_spans) return;
    const int j = (wi % per_span) / a.Hkv;
    const int kvh = wi % a.Hkv;
    const int len = a.ctx_len[j] + 1;
    const int k_begin = span * kSpan;
    if (k_begin >= len) return;
    const int k_end = min(len, k_begin + kSpan);
    const int col = lane & 15, g4 = lane >> 4;

    // The span's 16 page ids, one per lane, fetched once: no key/value load waits on a page-table read.  Ids that
    // are out of range or belong to pages past the end of the context are replaced by page 0: every load below
    // then has a valid address and no branch, and what it fetches for such a page is masked out.
    int my_page = 0;
    {
        const int lp = (k_begin >> 4) + col;
        if (lp * 16 < k_end && lp < a.max_pages) my_page = a.page_table[(size_t)j * a.max_pages + lp];
        if ((unsigned)my_page >= (unsigned)a.n_pages) my_page = 0;
    }

    int q_row = 0;
    if (a.lead_cu) {
        int tiles = j;
        for (int i = 0; i < a.n_lead; ++i) tiles += (a.lead_cu[i + 1] - a.lead_cu[i] + 31) >> 5;
        q_row = tiles * 32;
    }
    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        u32x4 v = {0, 0, 0, 0};
        if (col < G) {
            const int k = (kvh * G + col) * HD + (kk * 4 + g4) * 8;
            v = *(const u32x4 *)(a.q + (a.lead_cu ? p32_offset(q_row, k, a.Hq * HD) : (size_t)j * a.Hq * HD + k));
        }
        qf[kk] = *(bf16x8 *)&v;
    }
    f32x4 o_acc[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) o_acc[i][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // One pair = two pages (A, B) = 32 keys.  S^T is computed as two 16-row tiles: tile 1 takes slots 0..7 of page
    // A and of page B (tokens {0..3, 8..11}), tile 2 slots 8..15 (tokens {4..7, 12..15}); lane (col = query head,
    // g4) then holds the scores of tokens 8*(g4 % 2) .. +7 of page g4 / 2, exactly the 8 tokens of the V^T operand
    // it reads with one 16-byte load.
    struct PairRegs {
        u32x4 k1[KK], k2[KK], v[RT];
    };
    const int half_off = (col & 7) * 8 + g4 * 128;  // elements: slot (col % 8) of a tile's half, k-group g4
    auto load_pair = [&](PairRegs &r, int pp) {
        const int pageA = __builtin_amdgcn_readlane(my_page, 2 * pp), pageB = __builtin_amdgcn_readlane(my_page, 2 * pp + 1);
        // K operand row (lane % 16): rows 0..7 from page A, 8..15 from page B
        const bf16_t *kp = a.k_pool + ((size_t)(col < 8 ? pageA : pageB) * a.Hkv + kvh) * BLK + half_off;
        // V operand: lane group g4 reads page g4 / 2, token group g4 % 2, hd rows 16 i + col
        const bf16_t *vp = a.v_pool + ((size_t)(g4 < 2 ? pageA : pageB) * a.Hkv + kvh) * BLK + ((g4 & 1) * HD + col) * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            // K/V pages are read once per kv head: non-temporal loads, so the stream does not evict what the prefill
            // phase shares through L2
            r.k1[kk] = __builtin_nontemporal_load((const u32x4 *)(kp + kk * 512));
            r.k2[kk] = __builtin_nontemporal_load((const u32x4 *)(kp + kk * 512 + 64));
        }
#pragma unroll
        for (int i = 0; i < RT; ++i) r.v[i] = __builtin_nontemporal_load((const u32x4 *)(vp + i * 128));
    };
    auto compute_pair = [&](PairRegs &r, int pp) {
        f32x4 s1 = {0, 0, 0, 0}, s2 = {0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&r.k1[kk], qf[kk], s1, 0, 0, 0);
            s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&r.k2[kk], qf[kk], s2, 0, 0, 0);
        }
        // register e of s1 is key key0 + e, of s2 key key0 + 4 + e
        const int key0 = k_begin + 32 * pp + 16 * (g4 >> 1) + 8 * (g4 & 1);
        float sv[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sv[e] = s1[e] * a.scale_log2e;
            sv[4 + e] = s2[e] * a.scale_log2e;
        }
        const bool tail = k_begin + 32 * pp + 32 > k_end;  // uniform: only the last pair of a context
        if (tail) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sv[e] = key0 + e < k_end ? sv[e] : -INFINITY;
            // values past the end of the context may hold anything; their weight is 0 but 0 * NaN is not
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (key0 + e >= k_end) r.v[i][e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
        }
        float mx = m_run;
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, sv[e]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // the first key of the span is always valid, so mx is finite
        const float alpha = __builtin_amdgcn_exp2f(m_run - mx);
        m_run = mx;
        float rs = 0.f;
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = __builtin_amdgcn_exp2f(sv[e] - mx);
            rs += p;
            pf[e] = (__bf16)p;
        }
        l_run = l_run * alpha + rs;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
#pragma unroll
            for (int e = 0; e < 4; ++e) o_acc[i][e] *= alpha;
            o_acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&r.v[i], pf, o_acc[i], 0, 0, 0);
        }
    };

    // Two register sets: the loads of the next pair are in flight while the current pair is computed.  The steady
    // state loop has no branch around a prefetch: with one, the paths with and without the extra loads in flight
    // merge, and the compiler can only wait as if they had not been issued, i.e. for the prefetch itself.
    const int n_pairs = (k_end - k_begin + 31) >> 5;
    PairRegs r0, r1;
    load_pair(r0, 0);
    int pp = 0;
    for (; pp + 2 < n_pairs; pp += 2) {
        load_pair(r1, pp + 1);
        compute_pair(r0, pp);
        load_pair(r0, pp + 2);
        compute_pair(r1, pp + 1);
    }
    if (pp + 1 < n_pairs) {
        load_pair(r1, pp + 1);
        compute_pair(r0, pp);
        compute_pair(r1, pp + 1);
    } else {
        compute_pair(r0, pp);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (col >= G) return;
    // register e of o_acc[i] is hd = 16 i + 4 g4 + e
    const size_t item = ((size_t)j * a.Hkv + kvh) * a.max_spans + span;
    // stored normalised (an average of value rows, inside half's range whenever the values are) and in half: half
    // the bytes of an fp32 partial, at a rounding 4x finer than the bf16 the values came in; a span is never empty
    const float inv_l = 1.0f / l_run;
    f16_t *po = a.part_o + (item * G + col) * HD;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        uint2 o = {packh2(o_acc[i][0] * inv_l, o_acc[i][1] * inv_l), packh2(o_acc[i][2] * inv_l, o_acc[i][3] * inv_l)};
        *(uint2 *)(po + 16 * i + 4 * g4) = o;
    }
    if (g4 == 0) {
        float2 ml = {m_run, l_run};
        *(float2 *)(a.part_ml + (item * G + col) * 2) = ml;
    }
}

// Merge of the span results of one (request, query head): with w_s = 2^(m_s - m) l_s and o_s the span's normalised
// output, o = sum_s w_s o_s / sum_s w_s, spans taken in order.  One wavefront per (request, query head); output in P32 order for the O projection.
template <int HD, int G>
__global__ __launch_bounds__(64) void attn_merge_kernel(AttnDecodeArgs a) {
    const int j = blockIdx.x / a.Hq, hq = blockIdx.x % a.Hq;
    const int kvh = hq / G, col = hq % G, lane = threadIdx.x;
    const int len = a.ctx_len[j] + 1;
    const int n_spans = (len + kSpan - 1) / kSpan;
    const size_t item0 = ((size_t)j * a.Hkv + kvh) * a.max_spans;
    constexpr int EPL = HD / 64;
    float acc[EPL], m = -INFINITY, denom = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    // spans are taken 64 at a time: lane s holds the statistics of span base + s, so the loads of the partial
    // outputs do not wait on one another
    for (int base = 0; base < n_spans; base += 64) {
        const int s = base + lane;
        float2 ml = {-INFINITY, 0.f};
        if (s < n_spans) ml = *(const float2 *)(a.part_ml + ((item0 + s) * G + col) * 2);
        float cm = ml.x;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cm = fmaxf(cm, __shfl_xor(cm, o));
        const float m_new = fmaxf(m, cm);
        const float rescale = exp2f(m - m_new);  // 0 on the first chunk (m = -inf), spans are never empty
        const float wl = s < n_spans ? exp2f(ml.x - m_new) * ml.y : 0.f;  // weight of the span's normalised output
        float part = wl;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
        denom = denom * rescale + part;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= rescale;
        const int cnt = min(64, n_spans - base);
        // eight spans' rows at a time, fetched by loads that do not wait on one another; summed in span order
        for (int k0 = 0; k0 < cnt; k0 += 8) {
            uint32_t pv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                pv[u] = 0;
                if (k0 + u < cnt) {
                    const f16_t *po = a.part_o + ((item0 + base + k0 + u) * G + col) * HD + lane * EPL;
                    pv[u] = EPL == 2 ? *(const uint32_t *)po : (uint32_t)po[0];
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float wk = __shfl(wl, (k0 + u) & 63);  // rows past cnt were read as zero
                acc[0] += wk * h2f((f16_t)(pv[u] & 0xffffu));
                if (EPL == 2) acc[EPL - 1] += wk * h2f((f16_t)(pv[u] >> 16));
            }
        }
        m = m_new;
    }
    const float inv = 1.0f / denom;
    const int QKp = a.Hq * HD;
    f16_t *dst = a.out + p32_offset(a.out_row0 + j, hq * HD + lane * EPL, QKp);
    if (EPL == 2) {
        *(uint32_t *)dst = packh2(acc[0] * inv, acc[EPL - 1] * inv);
    } else {
        dst[0] = f2h(acc[0] * inv);
    }
}

}  // namespace nexus
