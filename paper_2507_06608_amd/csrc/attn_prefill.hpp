// Chunked-prefill attention (Eq. 4 with the causal bound): every chunk row at absolute position pos attends to
// keys 0..pos of its request -- the cached prefix and the causal part of the chunk -- read through the page table.
//
// One workgroup serves 32*SPB chunk tokens of one request for all G query heads of one KV head, so each K/V page
// is fetched once per KV head and shared by G*SPB wavefronts through LDS.  Each wavefront owns a 32-token strip of
// one query head and works on the transposed problem:
//     S^T[keys][tokens] = K * Q^T          (v_mfma_f32_32x32x16_bf16; K tile is operand A, Q^T operand B)
//     O^T[hd][tokens]  += V^T * P^T        (V^T operand A, P^T operand B)
// In that orientation a lane owns one token column: the softmax running max / sum are per-lane scalars, and the
// S^T accumulator registers of a lane are, as they stand, the P^T operand of the second product (registers
// 8p .. 8p+7 are tokens 8g .. 8g+7 of page p, the eight k-slots of that page's PV instruction), so the
// probabilities never leave registers.  The private page layouts make both LDS reads conflict-free 16-byte reads.
//
// K/V tiles of 32 keys (2 pages of K, 2 of V) move global->LDS asynchronously (global_load_lds_dwordx4, 1 KiB per
// wavefront instruction, page blocks copied verbatim) into a ring of stages: the tiles in flight, the tile whose K
// operands are read, and the two before it, whose V operands are read two iterations later.  The request's page ids
// are staged in LDS once so that no load waits on a page-table read.  A short chunk has too few (strip, head) pairs
// to fill the chip, so the key range can be split over gridDim.z workgroups whose partial (max, sum, O) results are
// merged by attn_prefill_merge_kernel; the split count depends on the problem only.
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
    f16_t *part_o;      // [n_splits][T][Hq][hd]   (n_splits > 1): each split's output normalised by its own sum, half
    float *part_ml;     // [n_splits][T][Hq][2]    its running max (log2 domain) and sum
    int T;
};

template <int N>
__device__ __forceinline__ void wait_vmcnt_attn() {  // s_waitcnt vmcnt(N) alone (gfx9 encoding)
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// key tiles [begin, end) of split z when n_tiles tiles are dealt to n_splits splits in contiguous runs
__device__ __forceinline__ void attn_split_range(int n_tiles, int n_splits, int z, int &begin, int &end) {
    const int per = (n_tiles + n_splits - 1) / n_splits;
    begin = z * per;
    end = begin + per < n_tiles ? begin + per : n_tiles;
}

constexpr int kAttnTile = 32;   // keys per LDS stage (2 pages of K and of V)
constexpr float kAttnLazyLog2 = 8.f;  // rise of a row's running maximum (log2 units) that moves the exponents' reference
// Tiles issued ahead of the one whose K operands are read.  The ring holds those, that one, and the two before it
// (V operands are read two iterations after the K operands).  A workgroup of up to four wavefronts shares its CU
// with a second one, and two rings of more than four 16 KiB stages would not fit the CU's LDS next to the staged
// page ids: it looks one tile ahead.
constexpr int attn_ahead(int n_waves) { return n_waves > 4 ? 3 : 1; }
constexpr int attn_stages(int n_waves) { return attn_ahead(n_waves) + 3; }

template <int HD, int G, int SPB>
__global__ __launch_bounds__(64 * G * SPB, 2) void attn_prefill_kernel(AttnPrefillArgs a) {  // two wavefronts per SIMD
    constexpr int NW = G * SPB;
    constexpr int BLK = kPage * HD * 2;      // bytes of one (page, kv head) block
    constexpr int UPB = BLK / 1024;          // 1 KiB units per block
    constexpr int STAGE = 4 * BLK;           // 2 K pages + 2 V pages = 32 keys
    constexpr int UNITS = 4 * UPB;
    constexpr int LW = NW >= 8 ? 8 : NW >= 4 ? 4 : NW;  // wavefronts that issue loads: UNITS / LW each
    static_assert(UNITS % LW == 0, "uniform load count per loading wavefront (the vmcnt waits rely on it)");
    constexpr int LPW = UNITS / LW;
    constexpr int NST = attn_stages(NW), AHEAD = attn_ahead(NW);
    constexpr int KK = HD / 16;              // k-steps of the QK^T product
    constexpr int RT = HD / 32;              // 32-row tiles of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int32_t *s_pt = (int32_t *)(smem + NST * STAGE);

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: branches on it are scalar branches
    const int hg = w % G, strip = w / G;
    const int g = lane >> 5, col = lane & 31;
    // The kv head is the fastest grid index: workgroups are dealt to the 8 XCDs round-robin, so with 8 kv heads
    // every query tile of a kv head runs on the same XCD and that head's K/V pages are fetched into one L2 instead
    // of all eight (with the tile index fastest, the 16 tiles of the benchmark chunk fetched 83 MB for 8 MB of K/V).
    const int kvh = blockIdx.x, z = blockIdx.z;
    const int r = blockIdx.y / a.tiles_per_req;
    const int lt = a.tiles_per_req - 1 - blockIdx.y % a.tiles_per_req;  // longest-running tiles first
    const int c0 = a.cu_chunk[r], n_r = a.cu_chunk[r + 1] - c0;
    if (lt * 32 * SPB >= n_r) return;
    int tile_base = 0;
    for (int i = 0; i < r; ++i) tile_base += (a.cu_chunk[i + 1] - a.cu_chunk[i] + 31) >> 5;
    const int prefix = a.prefix_len[r];
    const int32_t *pt = a.page_table + (size_t)r * a.max_pages;

    int blk_last = (lt + 1) * 32 * SPB;
    if (blk_last > n_r) blk_last = n_r;
    const int kmax = prefix + blk_last;            // keys [0, kmax) are visible to some row of this block
    const int n_kv_tiles = (kmax + kAttnTile - 1) / kAttnTile;
    int pages_valid = (kmax + 15) >> 4;
    if (pages_valid > a.max_pages) pages_valid = a.max_pages;
    if (pages_valid > kAttnMaxPages) pages_valid = kAttnMaxPages;
    int t_begin, t_end;
    attn_split_range(n_kv_tiles, a.n_splits, z, t_begin, t_end);
    if (t_begin >= t_end) return;  // the merge kernel applies the same rule and never reads this split

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

    // Page ids of the request, staged once.  Ids out of range become page 0: every load then has a valid address
    // (and every wavefront issues the same number of loads per tile); what such a page delivers is masked out.
    for (int i = tid; i < pages_valid; i += 64 * NW) {
        const int page = pt[i];
        s_pt[i] = (unsigned)page < (unsigned)a.n_pages ? page : 0;
    }
    // The query loads above are waited for here, once: inside the loop only the tile loads are then in flight,
    // and the counted waits on them are the only vector-memory waits the loop needs.
    wait_vmcnt_attn<0>();
    __syncthreads();

    f32x16 o_acc[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[i][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // unit u of a stage: block u / UPB (0, 1: K pages; 2, 3: V pages of the tile), KiB u % UPB of that block
    auto issue = [&](int tile) {
        if (w >= LW) return;
        char *dst = smem + (tile % NST) * STAGE;
        // the tile's two page ids, read once
        const int page_a = tile * 2 < pages_valid ? s_pt[tile * 2] : 0;
        const int page_b = tile * 2 + 1 < pages_valid ? s_pt[tile * 2 + 1] : 0;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int u = w + LW * i;
            const int which = u / UPB;
            const int page = (which & 1) ? page_b : page_a;
            const char *src = (const char *)((which < 2 ? a.k_pool : a.v_pool) + ((size_t)page * a.Hkv + kvh) * (kPage * HD)) +
                              (u % UPB) * 1024 + lane * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(dst + u * 1024), 16, 0, 0);
        }
    };

    // The loop is software-pipelined over the key tiles, three tiles deep in its steady state (see below): the
    // scores of tile t, the softmax of tile t - 1 and the PV product of tile t - 2 share an iteration.  Tiles that
    // need the causal mask or reach past the block's last key, and the first iteration, take the plain order
    // (softmax and PV of the pending tile, then the scores of the new one).
    f32x16 s;  // scores of the pending tile
    auto read_k = [&](const char *sK, bf16x8 (&kf)[KK]) __attribute__((always_inline)) {
        // operand A row (lane % 32): page row / 16, slot row % 16 (slots are rows as they stand); k-slot group g
        const char *kp = sK + (col >> 4) * BLK + (col & 15) * 16 + g * 256;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[kk] = *(const bf16x8 *)(kp + kk * 512);
    };
    auto read_v = [&](const char *sK, u32x4 (&vf)[2][RT]) __attribute__((always_inline)) {
        // V block [2 token groups][hd][8]: lane (col, g) reads hd row 32 i + col of token group g
        const char *sV = sK + 2 * BLK;
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int i = 0; i < RT; ++i) vf[pg][i] = *(const u32x4 *)(sV + pg * BLK + (g * HD + col) * 16 + i * 512);
    };
    // Softmax of the scores in s (tile `tile`) in two parts.  First the running maximum: returns the factor alpha the
    // output accumulators must be rescaled by before this tile's PV product, and the reference mref of the exponents.
    auto softmax_max = [&](int tile, const bool need_mask, float &mref) __attribute__((always_inline)) -> float {
        const int key0 = tile * kAttnTile;
        // Register 4b + j of s is row 8b + 4g + j: page b / 2, slot 8(b%2) + 4g + j, which holds token
        // 8g + 4(b%2) + j.  So registers 8p .. 8p+7 are tokens 8g .. 8g+7 of page p, in order.
        // The running maximum is kept in scaled units (score * log2(e) / sqrt(hd)); the scale is positive, so
        // the maximum is taken over the raw scores and scaled once, and the scaling of every score is folded
        // into the exponent's fused multiply-add.
        float mraw = -INFINITY;
        if (need_mask) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = key0 + 16 * (e >> 3) + 8 * g + (e & 7);
                s[e] = key <= pos ? s[e] : -INFINITY;
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) mraw = fmaxf(mraw, s[e]);
        float mx = fmaxf(m_run, mraw * a.scale_log2e);
        mx = xor32_max(mx);
        // The reference of the exponents follows the running maximum lazily: it moves only when the maximum has
        // risen by more than kAttnLazyLog2 since it was last set.  Any reference gives the same softmax as long as
        // sum and accumulators refer to the same one; a stale one lets the probabilities reach 2^kAttnLazyLog2
        // instead of 1 (no matter to fp32 sums or bf16 operands) and spares the rescale of the 16 RT accumulator
        // registers on almost every tile (with 32 rows a wavefront, some row sets a new maximum in most tiles of
        // the first few thousand keys).
        const float m_new = mx > m_run + kAttnLazyLog2 ? mx : m_run;
        // a row may see no key at all in this split's range yet: keep the arithmetic finite
        mref = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - mref);
        m_run = m_new;
        return alpha;
    };
    // Then the exponentials: s holds the probabilities afterwards, and the running sum moves on.
    auto softmax_exp = [&](float mref, float alpha) __attribute__((always_inline)) {
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], a.scale_log2e, -mref));
            s[e] = p;
            rs += p;
        }
        l_run = l_run * alpha + rs;
    };
    // O^T *= alpha.  After the first few tiles the maximum rarely moves and alpha is exactly 1 in every lane: the 16 RT
    // multiplications are then skipped (multiplying by 1.0 changes no bit).
    auto rescale = [&](float alpha) __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) o_acc[i][e] *= alpha;
        }
    };
    // the probabilities in s as the two bf16 operands of the PV product (token groups 0 and 1 of the tile)
    auto pack_p = [&](bf16x8 (&pf)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[pg][e] = (__bf16)s[8 * pg + e];
    };
    // O^T += V^T P^T
    auto pv = [&](const bf16x8 (&pf)[2], u32x4 (&vf)[2][RT]) __attribute__((always_inline)) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int i = 0; i < RT; ++i)
                o_acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(bf16x8 *)&vf[pg][i], pf[pg], o_acc[i], 0, 0, 0);
    };
    // the plain order for the pending tile: V operands, softmax, PV
    auto softmax_pv = [&](int tile) __attribute__((always_inline)) {
        const int key0 = tile * kAttnTile;
        u32x4 vf[2][RT];
        read_v(smem + (tile % NST) * STAGE, vf);
        float mref;
        const float alpha = softmax_max(tile, key0 + kAttnTile - 1 > wave_min_pos, mref);
        softmax_exp(mref, alpha);
        rescale(alpha);
        // V slots at or past kmax may hold anything (even NaN): their probability is exactly 0, but 0 * NaN is
        // not, so the last tile zeroes them.
        if (key0 + kAttnTile > kmax) {  // uniform: the last tile of the block only
#pragma unroll
            for (int pg = 0; pg < 2; ++pg) {
                const int left = kmax - (key0 + 16 * pg + 8 * g);  // tokens of this group that are valid
#pragma unroll
                for (int i = 0; i < RT; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e >= left) vf[pg][i][e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
            }
        }
        bf16x8 pf[2];
        pack_p(pf);
        pv(pf, vf);
    };

#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (t_begin + i < t_end) issue(t_begin + i);
    // what every wavefront does at the top of an iteration, whatever it computes there, in two steps
    auto tile_barrier = [&](int tile) __attribute__((always_inline)) {
        // loads issued after those of this tile and allowed to stay in flight: min(AHEAD - 1, tiles left after it)
        const int later = t_end - 1 - tile;
        if (later >= AHEAD - 1) wait_vmcnt_attn<(AHEAD - 1) * LPW>();
        else if (later == 1) wait_vmcnt_attn<LPW>();
        else wait_vmcnt_attn<0>();
        // Everyone's part of this tile has landed, and everyone has issued the matrix instructions that consume the
        // operands of tile - 3 (hence has them in registers): the stage of tile - 3 may be refilled.
        __builtin_amdgcn_s_barrier();
    };
    auto tile_refill = [&](int tile) __attribute__((always_inline)) {
        if (tile + AHEAD < t_end) issue(tile + AHEAD);
    };
    auto tile_landed = [&](int tile) __attribute__((always_inline)) {
        tile_barrier(tile);
        tile_refill(tile);
    };
    // the plain iteration: softmax and PV of the pending tile, then the scores of this one
    bool pending = false;  // s holds the scores of tile - 1, whose softmax and PV are still to come
    auto plain_iteration = [&](int tile) __attribute__((always_inline)) {
        tile_landed(tile);
        // rows of this wave see keys up to prefix + st*32 + 31; tiles entirely past that contribute nothing
        const bool act = wave_active && tile * kAttnTile <= wave_min_pos + 31;
        if (pending) softmax_pv(tile - 1);
        pending = act;
        if (act) {
            bf16x8 kf[KK];
            read_k(smem + (tile % NST) * STAGE, kf);
#pragma unroll
            for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
        }
    };
    // Interleaved iterations run for the tiles t whose predecessors need no mask (every key visible to every row of
    // this wavefront) and lie inside the block's key range: t_begin < t <= t_il, a range that depends on the
    // wavefront's strip.  Every wavefront passes one barrier per tile in either kind of iteration.
    int t_il = (wave_min_pos + 1) / kAttnTile;
    if (kmax / kAttnTile < t_il) t_il = kmax / kAttnTile;
    if (t_end - 1 < t_il) t_il = t_end - 1;
    if (!wave_active) t_il = t_begin;
    int tile = t_begin;
    plain_iteration(tile++);
    if (tile <= t_il) {
        // Three tiles in flight per wavefront: iteration t issues the QK^T chain of tile t and the PV product of tile
        // t - 2 (probabilities packed an iteration ago) as ONE run of 2 KK matrix instructions, and spreads the whole
        // softmax of tile t - 1 between them; nothing in the run depends on anything else in it.
        bf16x8 pf[2];        // probabilities of tile - 2 (after the filling iteration: of tile - 1)
        float alpha_pend;    // factor the accumulators take before that tile's PV product
        {   // filling iteration: scores of this tile, softmax of the pending one, no PV yet
            tile_landed(tile);
            bf16x8 kf[KK];
            read_k(smem + (tile % NST) * STAGE, kf);
            float mref;
            alpha_pend = softmax_max(tile - 1, false, mref);
            f32x16 sn;
#pragma unroll
            for (int e = 0; e < 16; ++e) sn[e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sn, 0, 0, 0);
            softmax_exp(mref, alpha_pend);
            pack_p(pf);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
            }
            s = sn;
            ++tile;
        }
        for (; tile <= t_il; ++tile) {
            tile_barrier(tile);
            bf16x8 kf[KK];
            u32x4 vf[2][RT];
            read_v(smem + ((tile - 2) % NST) * STAGE, vf);
            read_k(smem + (tile % NST) * STAGE, kf);
            // the refill (page ids out of LDS, addresses, loads) comes behind the operand reads: it works tiles ahead
            // and is in no hurry, the matrix unit waits for the operands
            tile_refill(tile);
            rescale(alpha_pend);
            // one scheduling region from here to the end of the iteration
            float mref;
            alpha_pend = softmax_max(tile - 1, false, mref);
            f32x16 sn;
#pragma unroll
            for (int e = 0; e < 16; ++e) sn[e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sn, 0, 0, 0);
            pv(pf, vf);
            softmax_exp(mref, alpha_pend);
            pack_p(pf);
#pragma unroll
            for (int i = 0; i < KK + 2 * RT; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
            }
            s = sn;
        }
        {   // draining: the PV product of tile - 2; its stage is still in the ring
            u32x4 vf[2][RT];
            read_v(smem + ((tile - 2) % NST) * STAGE, vf);
            rescale(alpha_pend);
            pv(pf, vf);
        }
    }
    for (; tile < t_end; ++tile) plain_iteration(tile);
    if (pending) softmax_pv(t_end - 1);

    if (!tok_ok) return;
    l_run += __shfl_xor(l_run, 32);  // both lanes of a column are valid together
    const int trow = c0 + local;
    // o_acc[i][4b + j] is hd = 32 i + 8 b + 4 g + j
    if (a.n_splits > 1) {
        // The partial output is stored normalised (an average of value rows, so within half's range whenever the
        // values are) and in half: half the bytes of an fp32 partial on the way out and into the merge, at a
        // rounding 4x finer than the bf16 the values came in.  A row that saw no key in this split stores zeros.
        const float inv_l = l_run > 0.f ? 1.0f / l_run : 0.f;
        f16_t *po = a.part_o + (((size_t)z * a.T + trow) * a.Hq + hq) * HD;
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                uint2 x = {packh2(o_acc[i][4 * b + 0] * inv_l, o_acc[i][4 * b + 1] * inv_l),
                           packh2(o_acc[i][4 * b + 2] * inv_l, o_acc[i][4 * b + 3] * inv_l)};
                *(uint2 *)(po + 32 * i + 8 * b + 4 * g) = x;
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
            uint2 o = {packh2(o_acc[i][4 * b + 0] * inv, o_acc[i][4 * b + 1] * inv), packh2(o_acc[i][4 * b + 2] * inv, o_acc[i][4 * b + 3] * inv)};
            *(uint2 *)(a.out + p32_offset(trow, hq * HD + 32 * i + 8 * b + 4 * g, QKp)) = o;
        }
}

// Merge of the key-range splits of one (token, query head): with w_z = 2^(m_z - m) l_z and o_z the split's normalised
// output, o = sum_z w_z o_z / sum_z w_z, the splits taken in order.  One wavefront per (token, head); a split is read only if the main kernel ran it.
constexpr int kAttnMaxSplits = 8;   // upper bound of the key-range split count (the merge unrolls over it)

// One wavefront per (token, group of 512 / HD consecutive query heads): a lane owns 8 consecutive head dimensions of
// one head, i.e. one 16-byte piece of each split's row and of the output row.
template <int HD, int SPB>
__global__ __launch_bounds__(64) void attn_prefill_merge_kernel(AttnPrefillArgs a) {
    constexpr int LPH = HD / 8;      // lanes per head
    constexpr int HPW = 64 / LPH;    // heads per wavefront
    const int lane = threadIdx.x;
    const int groups = (a.Hq + HPW - 1) / HPW;
    const int t = blockIdx.x / groups;
    const int hq = (blockIdx.x % groups) * HPW + lane / LPH, d0 = (lane % LPH) * 8;
    int r = 0;
    while (r + 1 < a.n_reqs && a.cu_chunk[r + 1] <= t) ++r;
    const int c0 = a.cu_chunk[r], n_r = a.cu_chunk[r + 1] - c0, local = t - c0;
    const int lt = local / (32 * SPB);
    int blk_last = (lt + 1) * 32 * SPB;
    if (blk_last > n_r) blk_last = n_r;
    const int n_kv_tiles = (a.prefix_len[r] + blk_last + kAttnTile - 1) / kAttnTile;
    if (hq >= a.Hq) return;
    // Every split's statistics, then every split's row, are fetched by loads that do not depend on one another
    // (the loops are unrolled over the largest split count): two memory latencies per output row, not one per split.
    float mz[kAttnMaxSplits], lz[kAttnMaxSplits];
#pragma unroll
    for (int z = 0; z < kAttnMaxSplits; ++z) {
        int b = 0, e = 0;
        if (z < a.n_splits) attn_split_range(n_kv_tiles, a.n_splits, z, b, e);
        float2 ml = {-INFINITY, 0.f};
        if (b < e) ml = *(const float2 *)(a.part_ml + (((size_t)z * a.T + t) * a.Hq + hq) * 2);
        mz[z] = ml.x, lz[z] = ml.y;
    }
    float m = -INFINITY;
#pragma unroll
    for (int z = 0; z < kAttnMaxSplits; ++z) m = fmaxf(m, mz[z]);  // split 0 always holds key 0, so m is finite
    u32x4 pz[kAttnMaxSplits];
#pragma unroll
    for (int z = 0; z < kAttnMaxSplits; ++z) {
        pz[z] = u32x4{0, 0, 0, 0};
        if (lz[z] > 0.f) pz[z] = *(const u32x4 *)(a.part_o + (((size_t)z * a.T + t) * a.Hq + hq) * HD + d0);
    }
    float acc[8], denom = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
    for (int z = 0; z < kAttnMaxSplits; ++z) {  // in split order
        const float wl = lz[z] > 0.f ? exp2f(mz[z] - m) * lz[z] : 0.f;
        denom += wl;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += wl * h2f((f16_t)(pz[z][i] & 0xffffu));
            acc[2 * i + 1] += wl * h2f((f16_t)(pz[z][i] >> 16));
        }
    }
    const float inv = 1.0f / denom;
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = packh2(acc[2 * i] * inv, acc[2 * i + 1] * inv);
    *(u32x4 *)(a.out + p32_offset(t, hq * HD + d0, a.Hq * HD)) = o;  // 8 consecutive k are contiguous in that layout
}

}  // namespace nexus
