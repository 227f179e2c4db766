// Chunked-prefill attention (Eq. 4 with the causal bound): every chunk row at absolute position pos attends to
// keys 0..pos of its request -- the cached prefix and the causal part of the chunk -- read through the page table.
//
// One workgroup serves 32*SPB chunk tokens of one request for all G query heads of one KV head, so each K/V page
// is fetched once per KV head and shared by G*SPB wavefronts through LDS.  Each wavefront owns a 32-token strip of
// one query head and works on the transposed problem:
//     S^T[keys][tokens] = K * Q^T          (v_mfma_f32_32x32x16_bf16; K tile is operand A, Q^T operand B)
//     O^T[hd][tokens]  += V^T * P^T        (V^T operand A, P^T operand B)
// In that orientation a lane owns one token column: the softmax running max / sum are per-lane scalars, and the
// S^T accumulator registers of a lane are, as they stand, the P^T operand of the second product (the register
// holding key 8b+4g+j of a 32-key group feeds k-slot 4(b%2)+j of the PV instruction of 16-key page b/2), so the
// probabilities never leave registers.  The private page layouts make both LDS reads conflict-free 16-byte reads.
//
// K/V tiles of 64 keys (4 pages of K, 4 of V) move global->LDS asynchronously (global_load_lds_dwordx4, 1 KiB per
// wavefront instruction, page blocks copied verbatim) into a two-stage ring; the request's page ids are staged in
// LDS once so that no load waits on a page-table read.  A short chunk has too few (strip, head) pairs to fill the
// chip, so the key range can be split over gridDim.z workgroups whose partial (max, sum, O) results are merged by
// attn_prefill_merge_kernel; the split count depends on the problem only.
#pragma once
#include "common.hpp"

namespace nexus {

constexpr int kAttnMaxPages = 2048;  // page ids staged in LDS per workgroup (32K tokens of context)

struct AttnPrefillArgs {
    const bf16_t *q;  // P32 [request-aligned rows][Hq*hd]
    f16_t *out;       // half, P32 [global token rows][Hq*hd] (operand of the output projection)
    const int32_t *cu_chunk, *prefix_len, *page_table;
    int n_reqs, max_pages, tiles_per_req;  // tiles of 32*SPB tokens sized from the max_chunk hint
    const bf16_t *k_pool, *v_pool;
    int n_pages, Hq, Hkv;
    float scale_log2e;  // log2(e) / sqrt(hd)
    int n_splits;       // gridDim.z
    float *part_o;      // [n_splits][T][Hq][hd]   (n_splits > 1)
    float *part_ml;     // [n_splits][T][Hq][2]
    int T;
};

// key tiles [begin, end) of split z when n_tiles tiles are dealt to n_splits splits in contiguous runs
__device__ __forceinline__ void attn_split_range(int n_tiles, int n_splits, int z, int &begin, int &end) {
    const int per = (n_tiles + n_splits - 1) / n_splits;
    begin = z * per;
    end = begin + per < n_tiles ? begin + per : n_tiles;
}

template <int HD, int G, int SPB>
__global__ __launch_bounds__(64 * G * SPB, 2) void attn_prefill_kernel(AttnPrefillArgs a) {  // two wavefronts per SIMD
    constexpr int NW = G * SPB;
    constexpr int BLK = kPage * HD * 2;      // bytes of one (page, kv head) block
    constexpr int UPB = BLK / 1024;          // 1 KiB units per block
    constexpr int STAGE = 8 * BLK;           // 4 K pages + 4 V pages = 64 keys
    constexpr int UNITS = 8 * UPB;
    constexpr int LPW = (UNITS + NW - 1) / NW;
    constexpr int KK = HD / 16;              // k-steps of the QK^T product
    constexpr int RT = HD / 64;              // pairs of 32-row tiles of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int32_t *s_pt = (int32_t *)(smem + 2 * STAGE);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int hg = w % G, strip = w / G;
    const int g = lane >> 5, col = lane & 31;
    const int kvh = blockIdx.y, z = blockIdx.z;
    const int r = blockIdx.x / a.tiles_per_req;
    const int lt = a.tiles_per_req - 1 - blockIdx.x % a.tiles_per_req;  // longest-running tiles first
    const int c0 = a.cu_chunk[r], n_r = a.cu_chunk[r + 1] - c0;
    if (lt * 32 * SPB >= n_r) return;
    int tile_base = 0;
    for (int i = 0; i < r; ++i) tile_base += (a.cu_chunk[i + 1] - a.cu_chunk[i] + 31) >> 5;
    const int prefix = a.prefix_len[r];
    const int32_t *pt = a.page_table + (size_t)r * a.max_pages;

    int blk_last = (lt + 1) * 32 * SPB;
    if (blk_last > n_r) blk_last = n_r;
    const int kmax = prefix + blk_last;            // keys [0, kmax) are visible to some row of this block
    const int n_kv_tiles = (kmax + 63) >> 6;
    int pages_valid = (kmax + 15) >> 4;
    if (pages_valid > a.max_pages) pages_valid = a.max_pages;
    if (pages_valid > kAttnMaxPages) pages_valid = kAttnMaxPages;
    int t_begin, t_end;
    attn_split_range(n_kv_tiles, a.n_splits, z, t_begin, t_end);
    if (t_begin >= t_end) return;  // the merge kernel applies the same rule and never reads this split

    for (int i = tid; i < pages_valid; i += 64 * NW) {
        const int page = pt[i];
        s_pt[i] = (unsigned)page < (unsigned)a.n_pages ? page : -1;
    }
    __syncthreads();

    const int st = lt * SPB + strip;               // this wave's 32-token strip inside the request
    const bool wave_active = st * 32 < n_r;
    const int local = st * 32 + col;
    const bool tok_ok = wave_active && local < n_r;
    const int pos = tok_ok ? prefix + local : 0x7fffffff;
    const int wave_min_pos = prefix + st * 32;

    const int hq = kvh * G + hg;
    const int QKp = a.Hq * HD;
    bf16x8 qf[KK];
    if (wave_active) {
        const bf16_t *qb = a.q + ((size_t)(tile_base + st) * (QKp >> 4) + (size_t)hq * KK) * 512 + lane * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk] = *(const bf16x8 *)(qb + kk * 512);
    } else {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[kk][e] = (__bf16)0.f;
    }

    f32x16 o_acc[RT][2];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int e = 0; e < 16; ++e) o_acc[i][p][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // unit u of a stage: block u / UPB (0..3 K pages, 4..7 V pages of the tile), KiB u % UPB of that block
    auto issue = [&](int tile) {
        char *dst = smem + (tile & 1) * STAGE;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int u = w + NW * i;
            if (u < UNITS) {
                const int which = u / UPB;
                const int lp = tile * 4 + (which & 3);
                if (lp < pages_valid) {
                    const int page = s_pt[lp];
                    if (page >= 0) {
                        const char *src = (const char *)((which < 4 ? a.k_pool : a.v_pool) + ((size_t)page * a.Hkv + kvh) * (kPage * HD)) +
                                          (u % UPB) * 1024 + lane * 16;
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                         (__attribute__((address_space(3))) void *)(dst + u * 1024), 16, 0, 0);
                    }
                }
            }
        }
    };

    issue(t_begin);
    for (int tile = t_begin; tile < t_end; ++tile) {
        const int cur = tile & 1;
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's part of the tile has landed
        __syncthreads();                     // everyone's part has landed; everyone is done with the other stage
        if (tile + 1 < t_end) issue(tile + 1);
        const int key0 = tile * 64;
        // rows of this wave see keys up to prefix + st*32 + 31; tiles entirely past that contribute nothing
        if (wave_active && key0 <= wave_min_pos + 31) {
            const char *sK = smem + cur * STAGE;
            const char *sV = sK + 4 * BLK;
            f32x16 s[2];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
#pragma unroll
                for (int e = 0; e < 16; ++e) s[h2][e] = 0.f;
                // operand A row (lane % 32) = key 32*h2 + row: page 2*h2 + row/16, token row%16; k-slot group g
                const char *kp = sK + (2 * h2 + (col >> 4)) * BLK + (col & 15) * 16 + g * 256;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    bf16x8 kf = *(const bf16x8 *)(kp + kk * 512);
                    s[h2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[h2], 0, 0, 0);
                }
            }
            // scale, causal mask (register 4b+j of group h2 is key key0 + 32*h2 + 8b + 4g + j), running max
            const bool need_mask = key0 + 63 > wave_min_pos;
            float mx = m_run;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float v = s[h2][e] * a.scale_log2e;
                    if (need_mask) {
                        const int key = key0 + 32 * h2 + 8 * (e >> 2) + 4 * g + (e & 3);
                        v = key <= pos ? v : -INFINITY;
                    }
                    s[h2][e] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // a row may see no key at all in this split's range yet: keep the arithmetic finite
            const float mref = mx == -INFINITY ? 0.f : mx;
            const float alpha = exp2f(m_run - mref);
            m_run = mx;
            float rs = 0.f;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = exp2f(s[h2][e] - mref);
                    s[h2][e] = p;
                    rs += p;
                }
            l_run = l_run * alpha + rs;
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int p = 0; p < 2; ++p)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o_acc[i][p][e] *= alpha;
            // V slots at or past kmax may hold anything (even NaN): their probability is exactly 0, but 0 * NaN is
            // not, so the last tile zeroes them as it reads them.
            const bool v_tail = key0 + 64 > kmax;
            // PV: page pg of the tile uses registers 8*(pg%2) .. +7 of group pg/2 as its 8 k-slots
#pragma unroll
            for (int pg = 0; pg < 4; ++pg) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s[pg >> 1][8 * (pg & 1) + e];
                // k-slot e<4 is token 4g+e, e>=4 is token 8+4g+(e-4): token groups g and g+2 of the page
                const char *vp = sV + pg * BLK + col * 16;
                uint32_t keep_lo = 0xffffffffu, keep_hi = 0xffffffffu, keep_lo2 = 0xffffffffu, keep_hi2 = 0xffffffffu;
                if (v_tail) {
                    // tokens of group g: key0 + 16 pg + 4 g + {0..3}; of group g + 2: eight further on
                    const int left = kmax - (key0 + 16 * pg + 4 * g);  // tokens of group g that are valid
                    const int left2 = left - 8;
                    keep_lo = left >= 2 ? 0xffffffffu : left == 1 ? 0x0000ffffu : 0u;   // tokens 0, 1
                    keep_hi = left >= 4 ? 0xffffffffu : left == 3 ? 0x0000ffffu : 0u;   // tokens 2, 3
                    keep_lo2 = left2 >= 2 ? 0xffffffffu : left2 == 1 ? 0x0000ffffu : 0u;
                    keep_hi2 = left2 >= 4 ? 0xffffffffu : left2 == 3 ? 0x0000ffffu : 0u;
                }
#pragma unroll
                for (int i = 0; i < RT; ++i) {
                    uint4 lo = *(const uint4 *)(vp + ((g)*HD + 64 * i) * 8);
                    uint4 hi = *(const uint4 *)(vp + ((g + 2) * HD + 64 * i) * 8);
                    if (v_tail) {
                        lo.x &= keep_lo, lo.y &= keep_hi, lo.z &= keep_lo, lo.w &= keep_hi;
                        hi.x &= keep_lo2, hi.y &= keep_hi2, hi.z &= keep_lo2, hi.w &= keep_hi2;
                    }
                    // each 16 B holds hd rows (64i + 2*col) and (64i + 2*col + 1), 4 tokens each
                    uint4 ev = make_uint4(lo.x, lo.y, hi.x, hi.y), od = make_uint4(lo.z, lo.w, hi.z, hi.w);
                    o_acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(bf16x8 *)&ev, pf, o_acc[i][0], 0, 0, 0);
                    o_acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(bf16x8 *)&od, pf, o_acc[i][1], 0, 0, 0);
                }
            }
        }
    }

    if (!tok_ok) return;
    l_run += __shfl_xor(l_run, 32);  // both lanes of a column are valid together
    const int trow = c0 + local;
    if (a.n_splits > 1) {
        // o_acc[i][par][4b+j] is hd = 64i + 16b + 8g + 2j + par: 8 consecutive floats per (i, b)
        float *po = a.part_o + (((size_t)z * a.T + trow) * a.Hq + hq) * HD;
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                float4 x0 = {o_acc[i][0][4 * b + 0], o_acc[i][1][4 * b + 0], o_acc[i][0][4 * b + 1], o_acc[i][1][4 * b + 1]};
                float4 x1 = {o_acc[i][0][4 * b + 2], o_acc[i][1][4 * b + 2], o_acc[i][0][4 * b + 3], o_acc[i][1][4 * b + 3]};
                *(float4 *)(po + 64 * i + 16 * b + 8 * g) = x0;
                *(float4 *)(po + 64 * i + 16 * b + 8 * g + 4) = x1;
            }
        if (g == 0) {
            float2 ml = {m_run, l_run};
            *(float2 *)(a.part_ml + (((size_t)z * a.T + trow) * a.Hq + hq) * 2) = ml;
        }
        return;
    }
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int hd0 = 64 * i + 16 * b + 8 * g;
            uint4 o = make_uint4(packh2(o_acc[i][0][4 * b + 0] * inv, o_acc[i][1][4 * b + 0] * inv),
                                 packh2(o_acc[i][0][4 * b + 1] * inv, o_acc[i][1][4 * b + 1] * inv),
                                 packh2(o_acc[i][0][4 * b + 2] * inv, o_acc[i][1][4 * b + 2] * inv),
                                 packh2(o_acc[i][0][4 * b + 3] * inv, o_acc[i][1][4 * b + 3] * inv));
            *(uint4 *)(a.out + p32_offset(trow, hq * HD + hd0, QKp)) = o;
        }
}

// Merge of the key-range splits of one (token, query head): o = sum_z 2^(m_z - m) o_z / sum_z 2^(m_z - m) l_z with
// the splits taken in order.  One wavefront per (token, head); a split is read only if the main kernel ran it.
template <int HD, int SPB>
__global__ __launch_bounds__(64) void attn_prefill_merge_kernel(AttnPrefillArgs a) {
    const int t = blockIdx.x / a.Hq, hq = blockIdx.x % a.Hq, lane = threadIdx.x;
    int r = 0;
    while (r + 1 < a.n_reqs && a.cu_chunk[r + 1] <= t) ++r;
    const int c0 = a.cu_chunk[r], n_r = a.cu_chunk[r + 1] - c0, local = t - c0;
    const int lt = local / (32 * SPB);
    int blk_last = (lt + 1) * 32 * SPB;
    if (blk_last > n_r) blk_last = n_r;
    const int n_kv_tiles = (a.prefix_len[r] + blk_last + 63) >> 6;
    float m = -INFINITY;
    for (int z = 0; z < a.n_splits; ++z) {
        int b, e;
        attn_split_range(n_kv_tiles, a.n_splits, z, b, e);
        if (b < e) m = fmaxf(m, a.part_ml[(((size_t)z * a.T + t) * a.Hq + hq) * 2]);
    }
    constexpr int EPL = HD / 64;
    float acc[EPL], denom = 0.f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    for (int z = 0; z < a.n_splits; ++z) {
        int b, e;
        attn_split_range(n_kv_tiles, a.n_splits, z, b, e);
        if (b >= e) continue;
        const size_t item = ((size_t)z * a.T + t) * a.Hq + hq;
        const float2 ml = *(const float2 *)(a.part_ml + item * 2);
        const float wgt = exp2f(ml.x - m);  // split 0 always holds key 0, so m is finite
        denom += wgt * ml.y;
        const float *po = a.part_o + item * HD + lane * EPL;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] += wgt * po[i];
    }
    const float inv = 1.0f / denom;
    f16_t *dst = a.out + p32_offset(t, hq * HD + lane * EPL, a.Hq * HD);
    if (EPL == 2) *(uint32_t *)dst = packh2(acc[0] * inv, acc[EPL - 1] * inv);
    else dst[0] = f2h(acc[0] * inv);
}

}  // namespace nexus
