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
// (S^T = K Q^T, O^T = V^T P^T) keeps softmax statistics per lane and lets the S^T accumulators of two pages
// serve directly as the P^T operand (k-slots 0..3 = page A tokens 4g..4g+3, k-slots 4..7 = page B).
#pragma once
#include "common.hpp"

namespace nexus {

constexpr int kSpan = 256;  // keys per work item (16 pages)

struct AttnDecodeArgs {
    const bf16_t *q;  // row-major [B][Hq*hd], rotated
    const int32_t *ctx_len, *page_table;
    int n_reqs, max_pages, max_spans;
    const bf16_t *k_pool, *v_pool;
    int n_pages, Hq, Hkv;
    float scale_log2e;
    float *part_o;   // [B][Hkv][max_spans][G][hd]
    float *part_ml;  // [B][Hkv][max_spans][G][2]  (running max in the log2 domain, sum)
    f16_t *out;      // merge output: half, P32 [B rows][Hq*hd]
};

template <int HD, int G>
__global__ __launch_bounds__(256, 2) void attn_decode_kernel(AttnDecodeArgs a) {
    constexpr int KK = HD / 32;   // k-steps of QK^T per page
    constexpr int RT = HD / 32;   // 32-row groups of O^T (two 16-row MFMA tiles each)
    constexpr int BLK = kPage * HD;  // elements per (page, kv head) block
    constexpr int NPAIR = kSpan / 32;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wi = blockIdx.x * 4 + w;
    const int span = wi % a.max_spans;
    const int kvh = (wi / a.max_spans) % a.Hkv;
    const int j = wi / (a.max_spans * a.Hkv);
    if (j >= a.n_reqs) return;
    const int len = a.ctx_len[j] + 1;
    const int k_begin = span * kSpan;
    if (k_begin >= len) return;
    const int k_end = min(len, k_begin + kSpan);
    const int col = lane & 15, g4 = lane >> 4;

    // the span's 16 page ids, one per lane, fetched once: no key/value load waits on a page-table read
    int my_page = -1;
    {
        const int lp = (k_begin >> 4) + col;
        if (lp * 16 < k_end && lp < a.max_pages) my_page = a.page_table[(size_t)j * a.max_pages + lp];
        if ((unsigned)my_page >= (unsigned)a.n_pages) my_page = -1;
    }

    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (col < G) v = *(const uint4 *)(a.q + (size_t)j * a.Hq * HD + (size_t)(kvh * G + col) * HD + (kk * 4 + g4) * 8);
        qf[kk] = *(bf16x8 *)&v;
    }
    f32x4 o_acc[RT][2];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int e = 0; e < 4; ++e) o_acc[i][p][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // One pair = two pages = 32 keys: 2 * KK key loads and 2 * RT value loads of 16 B per lane, all issued together.
    // V block [4 token groups][hd][4]: a lane reads hd rows 32i + 2*col, +1 of token group g4 (16 B).
    struct PairRegs {
        u32x4 ka[KK], kb[KK], va[RT], vb[RT];
    };
    auto load_pair = [&](PairRegs &r, int pp) {
        const int pageA = __builtin_amdgcn_readlane(my_page, 2 * pp), pageB = __builtin_amdgcn_readlane(my_page, 2 * pp + 1);
        const u32x4 zero = {0, 0, 0, 0};
        const bf16_t *kA = a.k_pool + ((size_t)(pageA < 0 ? 0 : pageA) * a.Hkv + kvh) * BLK;
        const bf16_t *kB = a.k_pool + ((size_t)(pageB < 0 ? 0 : pageB) * a.Hkv + kvh) * BLK;
        const bf16_t *vA = a.v_pool + ((size_t)(pageA < 0 ? 0 : pageA) * a.Hkv + kvh) * BLK;
        const bf16_t *vB = a.v_pool + ((size_t)(pageB < 0 ? 0 : pageB) * a.Hkv + kvh) * BLK;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            r.ka[kk] = pageA >= 0 ? *(const u32x4 *)(kA + kk * 512 + lane * 8) : zero;
            r.kb[kk] = pageB >= 0 ? *(const u32x4 *)(kB + kk * 512 + lane * 8) : zero;
        }
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            r.va[i] = pageA >= 0 ? *(const u32x4 *)(vA + (g4 * HD + 32 * i + 2 * col) * 4) : zero;
            r.vb[i] = pageB >= 0 ? *(const u32x4 *)(vB + (g4 * HD + 32 * i + 2 * col) * 4) : zero;
        }
    };
    auto compute_pair = [&](PairRegs &r, int pp) {
        f32x4 sA = {0, 0, 0, 0}, sB = {0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&r.ka[kk], qf[kk], sA, 0, 0, 0);
            sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&r.kb[kk], qf[kk], sB, 0, 0, 0);
        }
        // lane (col = query head, g4): register e of sA is key keyA + e, of sB key keyA + 16 + e
        const int keyA = k_begin + 32 * pp + 4 * g4, keyB = keyA + 16;
        float mx = m_run;
        float sv[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sv[e] = (keyA + e < k_end) ? sA[e] * a.scale_log2e : -INFINITY;
            sv[4 + e] = (keyB + e < k_end) ? sB[e] * a.scale_log2e : -INFINITY;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, sv[e]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // the first key of the span is always valid, so mx is finite
        const float alpha = exp2f(m_run - mx);
        m_run = mx;
        float rs = 0.f;
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = exp2f(sv[e] - mx);
            rs += p;
            pf[e] = (__bf16)p;
        }
        l_run = l_run * alpha + rs;
        // values past the end of the context may hold anything; their weight is 0 but 0 * NaN is not
        if (keyB + 4 > k_end) {
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t keep = (e & 1) ? 0x0000ffffu : 0xffff0000u;
                    if (keyA + (e & 3) >= k_end) r.va[i][e >> 1] &= keep;
                    if (keyB + (e & 3) >= k_end) r.vb[i][e >> 1] &= keep;
                }
        }
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            // 16 B = [hd row even: 4 tokens][hd row odd: 4 tokens]; operand A k-slots 0..3 from page A, 4..7 from page B
            u32x4 ev = {r.va[i][0], r.va[i][1], r.vb[i][0], r.vb[i][1]}, od = {r.va[i][2], r.va[i][3], r.vb[i][2], r.vb[i][3]};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o_acc[i][0][e] *= alpha;
                o_acc[i][1][e] *= alpha;
            }
            o_acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&ev, pf, o_acc[i][0], 0, 0, 0);
            o_acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&od, pf, o_acc[i][1], 0, 0, 0);
        }
    };

    // two register sets: the loads of the next pair are in flight while the current pair is computed
    const int n_pairs = (k_end - k_begin + 31) >> 5;
    PairRegs r0, r1;
    load_pair(r0, 0);
#pragma unroll
    for (int pp = 0; pp < NPAIR; pp += 2) {
        if (pp >= n_pairs) break;
        if (pp + 1 < n_pairs) load_pair(r1, pp + 1);
        compute_pair(r0, pp);
        if (pp + 1 >= n_pairs) break;
        if (pp + 2 < n_pairs) load_pair(r0, pp + 2);
        compute_pair(r1, pp + 1);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (col >= G) return;
    // o_acc[i][par][e] is hd = 32i + 2*(4*g4 + e) + par  ->  8 consecutive floats from hd0 = 32i + 8*g4
    const size_t item = ((size_t)j * a.Hkv + kvh) * a.max_spans + span;
    float *po = a.part_o + (item * G + col) * HD;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        float4 lo = {o_acc[i][0][0], o_acc[i][1][0], o_acc[i][0][1], o_acc[i][1][1]};
        float4 hi = {o_acc[i][0][2], o_acc[i][1][2], o_acc[i][0][3], o_acc[i][1][3]};
        *(float4 *)(po + 32 * i + 8 * g4) = lo;
        *(float4 *)(po + 32 * i + 8 * g4 + 4) = hi;
    }
    if (g4 == 0) {
        float2 ml = {m_run, l_run};
        *(float2 *)(a.part_ml + (item * G + col) * 2) = ml;
    }
}

// Merge of the span results of one (request, query head): o = sum_s 2^(m_s - m) o_s / sum_s 2^(m_s - m) l_s,
// spans taken in order.  One wavefront per (request, query head); output in P32 order for the O projection.
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
        const float wgt = s < n_spans ? exp2f(ml.x - m_new) : 0.f;
        float part = wgt * ml.y;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
        denom = denom * rescale + part;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= rescale;
        const int cnt = min(64, n_spans - base);
        for (int k = 0; k < cnt; ++k) {
            const float wk = __shfl(wgt, k);
            const float *po = a.part_o + ((item0 + base + k) * G + col) * HD + lane * EPL;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += wk * po[e];
        }
        m = m_new;
    }
    const float inv = 1.0f / denom;
    const int QKp = a.Hq * HD;
    f16_t *dst = a.out + p32_offset(j, hq * HD + lane * EPL, QKp);
    if (EPL == 2) {
        *(uint32_t *)dst = packh2(acc[0] * inv, acc[EPL - 1] * inv);
    } else {
        dst[0] = f2h(acc[0] * inv);
    }
}

}  // namespace nexus
