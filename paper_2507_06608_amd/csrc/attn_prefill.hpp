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
#pragma once
#include "common.hpp"

namespace nexus {

struct AttnPrefillArgs {
    const bf16_t *q;  // P32 [request-aligned rows][Hq*hd]
    bf16_t *out;      // P32 [global token rows][Hq*hd]
    const int32_t *cu_chunk, *prefix_len, *page_table;
    int n_reqs, max_pages, tiles_per_req;  // tiles of 32*SPB tokens sized from the max_chunk hint
    const bf16_t *k_pool, *v_pool;
    int n_pages, Hq, Hkv;
    float scale_log2e;  // log2(e) / sqrt(hd)
};

template <int HD, int G, int SPB>
__global__ __launch_bounds__(64 * G * SPB) void attn_prefill_kernel(AttnPrefillArgs a) {
    constexpr int NW = G * SPB, NT = 64 * NW;
    constexpr int BLK = kPage * HD * 2;      // bytes of one (page, kv head) block
    constexpr int STAGE = 8 * BLK;           // 4 K pages + 4 V pages = 64 keys
    constexpr int CHUNKS = STAGE / 16;       // 16-byte chunks per stage
    constexpr int CPT = (CHUNKS + NT - 1) / NT;
    constexpr int KK = HD / 16;              // k-steps of the QK^T product
    constexpr int RT = HD / 64;              // pairs of 32-row tiles of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int hg = w % G, strip = w / G;
    const int g = lane >> 5, col = lane & 31;
    const int kvh = blockIdx.y;
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
    const int pages_valid = (kmax + 15) >> 4;

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

    // ---- stage loader: chunk c of a stage = block (c / (BLK/16)) [0..3 K pages, 4..7 V pages], 16 B at c % (BLK/16)
    uint4 regs[CPT];
    auto load_tile = [&](int tile) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * NT;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (c < CHUNKS) {
                const int which = c / (BLK / 16), off = c % (BLK / 16);
                const int lp = tile * 4 + (which & 3);
                if (lp < pages_valid && lp < a.max_pages) {
                    const int page = pt[lp];
                    if ((unsigned)page < (unsigned)a.n_pages) {
                        const bf16_t *base = (which < 4 ? a.k_pool : a.v_pool) + ((size_t)page * a.Hkv + kvh) * (kPage * HD);
                        v = *(const uint4 *)((const char *)base + off * 16);
                        if (which >= 4 && lp * 16 + 16 > kmax) {
                            // V slots at or past kmax may hold anything (even NaN); their probability is exactly 0
                            // but 0 * NaN is not.  Zero them.  16 B = 2 hd rows x 4 tokens of group off / (HD/2).
                            const int kg = off / (HD / 2);
                            const int first_bad = kmax - (lp * 16 + kg * 4);  // tokens >= first_bad are invalid
                            uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if ((e & 3) >= first_bad) wds[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                            v = make_uint4(wds[0], wds[1], wds[2], wds[3]);
                        }
                    }
                }
            }
            regs[i] = v;
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * NT;
            if (c < CHUNKS) *(uint4 *)(smem + buf * STAGE + c * 16) = regs[i];
        }
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int tile = 0; tile < n_kv_tiles; ++tile) {
        const int cur = tile & 1;
        const bool more = tile + 1 < n_kv_tiles;
        if (more) load_tile(tile + 1);
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
            // key 0 is visible to every valid row, so mx is finite from the first tile on
            const float alpha = exp2f(m_run - mx);
            m_run = mx;
            float rs = 0.f;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = exp2f(s[h2][e] - mx);
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
            // PV: page pg of the tile uses registers 8*(pg%2) .. +7 of group pg/2 as its 8 k-slots
#pragma unroll
            for (int pg = 0; pg < 4; ++pg) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s[pg >> 1][8 * (pg & 1) + e];
                // k-slot e<4 is token 4g+e, e>=4 is token 8+4g+(e-4): token groups g and g+2 of the page
                const char *vp = sV + pg * BLK + col * 16;
#pragma unroll
                for (int i = 0; i < RT; ++i) {
                    const uint4 lo = *(const uint4 *)(vp + ((g)*HD + 64 * i) * 8);
                    const uint4 hi = *(const uint4 *)(vp + ((g + 2) * HD + 64 * i) * 8);
                    // each 16 B holds hd rows (64i + 2*col) and (64i + 2*col + 1), 4 tokens each
                    uint4 ev = make_uint4(lo.x, lo.y, hi.x, hi.y), od = make_uint4(lo.z, lo.w, hi.z, hi.w);
                    o_acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(bf16x8 *)&ev, pf, o_acc[i][0], 0, 0, 0);
                    o_acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(bf16x8 *)&od, pf, o_acc[i][1], 0, 0, 0);
                }
            }
        }
        if (more) store_tile(cur ^ 1);
        __syncthreads();
    }

    if (!tok_ok) return;
    l_run += __shfl_xor(l_run, 32);  // both lanes of a column are valid together
    const float inv = 1.0f / l_run;
    // o_acc[i][par][4b+j] is hd = 64i + 2*(8b+4g+j) + par: for fixed (i, b) a lane holds 8 consecutive hd
    bf16_t *ob = a.out;
    const int trow = c0 + local;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int hd0 = 64 * i + 16 * b + 8 * g;
            uint4 o = make_uint4(pack2(o_acc[i][0][4 * b + 0] * inv, o_acc[i][1][4 * b + 0] * inv),
                                 pack2(o_acc[i][0][4 * b + 1] * inv, o_acc[i][1][4 * b + 1] * inv),
                                 pack2(o_acc[i][0][4 * b + 2] * inv, o_acc[i][1][4 * b + 2] * inv),
                                 pack2(o_acc[i][0][4 * b + 3] * inv, o_acc[i][1][4 * b + 3] * inv));
            *(uint4 *)(ob + p32_offset(trow, hq * HD + hd0, QKp)) = o;
        }
}

}  // namespace nexus
