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
    bf16_t *out;     // merge output: P32 [B rows][Hq*hd]
};

template <int HD, int G>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnDecodeArgs a) {
    constexpr int KK = HD / 32;   // k-steps of QK^T per page
    constexpr int RT = HD / 32;   // 32-row groups of O^T (two 16-row MFMA tiles each)
    constexpr int BLK = kPage * HD;  // elements per (page, kv head) block
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
    const int32_t *pt = a.page_table + (size_t)j * a.max_pages;

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

    const int n_pairs = (k_end - k_begin + 31) >> 5;
    for (int pp = 0; pp < n_pairs; ++pp) {
        const int lpA = (k_begin >> 4) + 2 * pp, lpB = lpA + 1;
        int pageA = -1, pageB = -1;
        if (lpA < a.max_pages) pageA = pt[lpA];
        if (lpB * 16 < k_end && lpB < a.max_pages) pageB = pt[lpB];
        const bool okA = (unsigned)pageA < (unsigned)a.n_pages, okB = (unsigned)pageB < (unsigned)a.n_pages;
        const bf16_t *kA = a.k_pool + ((size_t)(okA ? pageA : 0) * a.Hkv + kvh) * BLK;
        const bf16_t *kB = a.k_pool + ((size_t)(okB ? pageB : 0) * a.Hkv + kvh) * BLK;
        const bf16_t *vA = a.v_pool + ((size_t)(okA ? pageA : 0) * a.Hkv + kvh) * BLK;
        const bf16_t *vB = a.v_pool + ((size_t)(okB ? pageB : 0) * a.Hkv + kvh) * BLK;

        // issue every load of the pair up front: 2 * KK key loads and 2 * RT value loads of 16 B per lane
        uint4 kfa[KK], kfb[KK], vfa[RT], vfb[RT];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            kfa[kk] = okA ? *(const uint4 *)(kA + kk * 512 + lane * 8) : make_uint4(0, 0, 0, 0);
            kfb[kk] = okB ? *(const uint4 *)(kB + kk * 512 + lane * 8) : make_uint4(0, 0, 0, 0);
        }
        // V block [4 token groups][hd][4]: lane reads hd rows 32i + 2*col, +1 of token group g4 (16 B)
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            vfa[i] = okA ? *(const uint4 *)(vA + (g4 * HD + 32 * i + 2 * col) * 4) : make_uint4(0, 0, 0, 0);
            vfb[i] = okB ? *(const uint4 *)(vB + (g4 * HD + 32 * i + 2 * col) * 4) : make_uint4(0, 0, 0, 0);
        }

        f32x4 sA = {0, 0, 0, 0}, sB = {0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&kfa[kk], qf[kk], sA, 0, 0, 0);
            sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&kfb[kk], qf[kk], sB, 0, 0, 0);
        }
        // lane (col = query head, g4): register e of sA is key lpA*16 + 4*g4 + e
        const int keyA = lpA * 16 + 4 * g4, keyB = keyA + 16;
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
        if (keyA + 4 > k_end || keyB + 4 > k_end || lpA * 16 + 32 > k_end) {
#pragma unroll
            for (int i = 0; i < RT; ++i) {
                uint32_t wa[4] = {vfa[i].x, vfa[i].y, vfa[i].z, vfa[i].w}, wb[4] = {vfb[i].x, vfb[i].y, vfb[i].z, vfb[i].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t keep = (e & 1) ? 0x0000ffffu : 0xffff0000u;
                    if (keyA + (e & 3) >= k_end) wa[e >> 1] &= keep;
                    if (keyB + (e & 3) >= k_end) wb[e >> 1] &= keep;
                }
                vfa[i] = make_uint4(wa[0], wa[1], wa[2], wa[3]);
                vfb[i] = make_uint4(wb[0], wb[1], wb[2], wb[3]);
            }
        }
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            // 16 B = [hd row even: 4 tokens][hd row odd: 4 tokens]; operand A k-slots 0..3 from page A, 4..7 from page B
            uint4 ev = make_uint4(vfa[i].x, vfa[i].y, vfb[i].x, vfb[i].y), od = make_uint4(vfa[i].z, vfa[i].w, vfb[i].z, vfb[i].w);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o_acc[i][0][e] *= alpha;
                o_acc[i][1][e] *= alpha;
            }
            o_acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&ev, pf, o_acc[i][0], 0, 0, 0);
            o_acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&od, pf, o_acc[i][1], 0, 0, 0);
        }
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
    float m = -INFINITY;
    for (int s = 0; s < n_spans; ++s) m = fmaxf(m, a.part_ml[((item0 + s) * G + col) * 2]);
    constexpr int EPL = HD / 64;
    float acc[EPL], denom = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int s = 0; s < n_spans; ++s) {
        const float2 ml = *(const float2 *)(a.part_ml + ((item0 + s) * G + col) * 2);
        const float wgt = exp2f(ml.x - m);
        denom += wgt * ml.y;
        const float *po = a.part_o + ((item0 + s) * G + col) * HD + lane * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += wgt * po[e];
    }
    const float inv = 1.0f / denom;
    const int QKp = a.Hq * HD;
    bf16_t *dst = a.out + p32_offset(j, hq * HD + lane * EPL, QKp);
    if (EPL == 2) {
        *(uint32_t *)dst = pack2(acc[0] * inv, acc[EPL - 1] * inv);
    } else {
        dst[0] = f2bf(acc[0] * inv);
    }
}

}  // namespace nexus
