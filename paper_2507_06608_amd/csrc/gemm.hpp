// MFMA projection GEMMs of the layer (Eq. 1-3): Y[T][N] = X[T][K] * W[N][K]^T with fused epilogues.  Operands are
// IEEE half (same matrix-unit rate as bfloat16, 8x smaller operand rounding), accumulation is fp32.
//
// Both operands are stored in P32 tile order (common.hpp), so every global access of the main loop is a
// contiguous 16 B per lane and the LDS image of a tile is the MFMA register image.  The kernel computes the
// transposed product Y^T = W * X^T: the weight tile is the MFMA "A" operand and the activation tile the "B"
// operand, which leaves each lane holding one token (column) and four consecutive features per register quad --
// the shape every epilogue wants (8-byte stores along the feature axis, rotary pairs and gate/up pairs in one
// lane).
//
// Reduction order depends only on (K, split count): never on the CU share the kernel runs on, so a phase
// produces bit-identical results alone, serialized or concurrent.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace nexus {

enum GemmEpi : int {
    EPI_ROWMAJOR = 0,  // out[t][f] = half(acc (+ bias[f]))                      (QKV projection)
    EPI_RES_IN = 1,    // out_f32[t][f] = bf16 res[t][f] + acc                   (x1 = x + attention projection)
    EPI_SWIGLU = 2,    // each weight strip = 16 gate rows + their 16 up rows; out_p32[t][f] = half(silu(gate) * up)
    EPI_PARTIAL = 3,   // partial[z][t][n] = acc (fp32), finished by splitk_reduce
    EPI_RES_OUT = 4    // out[t][f] = bf16(res_f32[t][f] + acc)                  (y = x1 + down projection)
};

struct GemmArgs {
    const f16_t *W;    // P32 [n_ftiles*32][Kp]
    const f16_t *X;    // P32 [n_ttiles*32][Kp]
    int n_ftiles, n_ttiles, Kp;
    int ksteps_per_split;  // K steps of 64 handled by one z-slice
    int T, N;              // valid tokens; N = n_ftiles * 32 (packed row count)
    void *out;             // row-major [T][ld_out]: half (ROWMAJOR), fp32 (RES_IN) or bf16 (RES_OUT)
    const void *res;       // row-major [T][ld_out]: bf16 (RES_IN) or fp32 (RES_OUT)
    const bf16_t *bias;    // [N] or null
    int ld_out;
    f16_t *out_p32;        // EPI_SWIGLU destination, P32 with out_Kp
    int out_Kp;
    float *partial;        // [S][T][N]
    int n_tblk;            // token blocks in the grid
    int n_xcd;             // XCDs the launch is spread over (tile-order remap), >= 1
    int group_f;           // feature blocks per tile group (tile-order remap inside an XCD), >= 1
};

constexpr int kGemmBK = 64;  // unit of the split-K bookkeeping: ksteps_per_split counts 64-wide k steps

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// ---- epilogue shared by the GEMM kernels -----------------------------------------------------------------------
// acc[i][j] is the 32x32 tile of feature strip (ft0 + i) x token strip (tt0 + j); the lane owns token column
// (lane % 32) and register 4*b + e is feature row 8*b + 4*(lane/32) + e.
template <int FW, int TW, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, f32x16 (&acc)[FW][TW], int ft0, int tt0, int z, int lane) {
    const int g = lane >> 5;
#pragma unroll
    for (int j = 0; j < TW; ++j) {
        const int t = (tt0 + j) * 32 + (lane & 31);
        if (t >= a.T) continue;
        if constexpr (EPI == EPI_SWIGLU) {
            // packed strip s = gate features [16 s, 16 s + 16) in rows 0..15, their up features in rows 16..31:
            // register quads b and b + 2 of one lane are a gate quad and its up quad
#pragma unroll
            for (int i = 0; i < FW; ++i) {
                const int ft = ft0 + i;
                if (ft >= a.n_ftiles) continue;
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int f = ft * 16 + 8 * b + 4 * g;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = silu_f(acc[i][j][4 * b + e]) * acc[i][j][4 * (b + 2) + e];
                    uint2 o = {packh2(v[0], v[1]), packh2(v[2], v[3])};
                    *(uint2 *)(a.out_p32 + p32_offset(t, f, a.out_Kp)) = o;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < FW; ++i) {
                const int ft = ft0 + i;
                if (ft >= a.n_ftiles) continue;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int f = ft * 32 + 8 * b + 4 * g;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * b + e];
                    if constexpr (EPI == EPI_PARTIAL) {
                        float4 o = {v[0], v[1], v[2], v[3]};
                        *(float4 *)(a.partial + ((size_t)z * a.T + t) * a.N + f) = o;
                    } else if constexpr (EPI == EPI_ROWMAJOR) {
                        if (a.bias) {
                            uint2 bb = *(const uint2 *)(a.bias + f);
                            v[0] += bf2f(bb.x & 0xffff), v[1] += bf2f(bb.x >> 16);
                            v[2] += bf2f(bb.y & 0xffff), v[3] += bf2f(bb.y >> 16);
                        }
                        uint2 o = {packh2(v[0], v[1]), packh2(v[2], v[3])};
                        *(uint2 *)((f16_t *)a.out + (size_t)t * a.ld_out + f) = o;
                    } else if constexpr (EPI == EPI_RES_IN) {
                        uint2 rr = *(const uint2 *)((const bf16_t *)a.res + (size_t)t * a.ld_out + f);
                        float4 o = {v[0] + bf2f(rr.x & 0xffff), v[1] + bf2f(rr.x >> 16), v[2] + bf2f(rr.y & 0xffff), v[3] + bf2f(rr.y >> 16)};
                        *(float4 *)((float *)a.out + (size_t)t * a.ld_out + f) = o;
                    } else {
                        float4 rr = *(const float4 *)((const float *)a.res + (size_t)t * a.ld_out + f);
                        uint2 o = {pack2(v[0] + rr.x, v[1] + rr.y), pack2(v[2] + rr.z, v[3] + rr.w)};
                        *(uint2 *)((bf16_t *)a.out + (size_t)t * a.ld_out + f) = o;
                    }
                }
            }
        }
    }
}

// The row-major epilogues (activations out, residual in, residual out, split-K partial sums) of the tiled GEMM, through LDS.  In the
// accumulators a lane owns a token column and 4 consecutive features per register quad: stored as they stand, one
// instruction puts 16 or 32 bytes into each of 32 different rows (and reads the residual the same way).  Here a
// wavefront first lays a 32-token x 64-feature block of its accumulators into its own LDS scratch, token-major,
// and then walks it row by row: 16 lanes cover the 64 features of a token, 4 features each, so the residual is
// read and the result written in whole 128- or 256-byte runs.  Same values, same arithmetic, other lanes.
// `scratch` is the wavefront's own kEpiScratch bytes; the workgroup has passed a barrier since its last operand read.
constexpr int kEpiPitch = 68;                        // floats per token row: 64 + 4 (the column writes spread over the banks)
constexpr int kEpiScratch = 32 * kEpiPitch * 4;      // bytes per wavefront
template <int FW, int TW, int EPI>
__device__ __forceinline__ void gemm_epilogue_rows(const GemmArgs &a, f32x16 (&acc)[FW][TW], int ft0, int tt0, int z, int lane, char *scratch) {
    static_assert(EPI == EPI_ROWMAJOR || EPI == EPI_RES_IN || EPI == EPI_RES_OUT || EPI == EPI_PARTIAL, "row-major epilogues only");
    float *sc = (float *)scratch;
    const int g = lane >> 5, col = lane & 31;
#pragma unroll
    for (int j = 0; j < TW; ++j) {
#pragma unroll
        for (int i0 = 0; i0 < FW; i0 += 2) {
            const int nfs = FW - i0 >= 2 ? 2 : 1;  // feature strips in this block
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                if (ii >= nfs) break;
                const int i = i0 + ii < FW ? i0 + ii : FW - 1;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float4 v = {acc[i][j][4 * b], acc[i][j][4 * b + 1], acc[i][j][4 * b + 2], acc[i][j][4 * b + 3]};
                    *(float4 *)(sc + col * kEpiPitch + ii * 32 + 8 * b + 4 * g) = v;
                }
            }
            // LDS serves a wavefront's requests in order: the reads below see the writes above
            const int cpt = nfs * 8;  // 4-feature chunks per token
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (k >= 4 * nfs) break;
                const int idx = lane + 64 * k;
                const int tok = idx / cpt, fc = idx % cpt;
                const float4 v = *(const float4 *)(sc + tok * kEpiPitch + fc * 4);
                const int t = (tt0 + j) * 32 + tok;
                const int ft = ft0 + i0 + (fc >> 3);
                if (t >= a.T || ft >= a.n_ftiles) continue;
                const int f = ft * 32 + (fc & 7) * 4;
                if constexpr (EPI == EPI_PARTIAL) {
                    *(float4 *)(a.partial + ((size_t)z * a.T + t) * a.N + f) = v;
                } else if constexpr (EPI == EPI_ROWMAJOR) {
                    float w[4] = {v.x, v.y, v.z, v.w};
                    if (a.bias) {
                        const uint2 bb = *(const uint2 *)(a.bias + f);
                        w[0] += bf2f(bb.x & 0xffff), w[1] += bf2f(bb.x >> 16);
                        w[2] += bf2f(bb.y & 0xffff), w[3] += bf2f(bb.y >> 16);
                    }
                    const uint2 o = {packh2(w[0], w[1]), packh2(w[2], w[3])};
                    *(uint2 *)((f16_t *)a.out + (size_t)t * a.ld_out + f) = o;
                } else if constexpr (EPI == EPI_RES_IN) {
                    const uint2 rr = *(const uint2 *)((const bf16_t *)a.res + (size_t)t * a.ld_out + f);
                    const float4 o = {v.x + bf2f(rr.x & 0xffff), v.y + bf2f(rr.x >> 16), v.z + bf2f(rr.y & 0xffff), v.w + bf2f(rr.y >> 16)};
                    *(float4 *)((float *)a.out + (size_t)t * a.ld_out + f) = o;
                } else {
                    const float4 rr = *(const float4 *)((const float *)a.res + (size_t)t * a.ld_out + f);
                    const uint2 o = {pack2(v.x + rr.x, v.y + rr.y), pack2(v.z + rr.z, v.w + rr.w)};
                    *(uint2 *)((bf16_t *)a.out + (size_t)t * a.ld_out + f) = o;
                }
            }
        }
    }
}

// s_waitcnt on the vector-memory counter alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters
// left at their maxima).  Asynchronous global->LDS loads are tracked by this counter.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

template <int N>
__device__ __forceinline__ void wait_lgkmcnt() {  // s_waitcnt lgkmcnt(N) alone (LDS / scalar-memory counter, 4 bits)
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
    __builtin_amdgcn_s_waitcnt(0xc07f | (N << 8));
}

// ---- main GEMM: asynchronous global->LDS tile loads, NST-stage ring --------------------------------------------
// A stage holds BKT k-tiles (16 k each) of FS weight strips and TS token strips, as 1 KiB units in P32 order.
// The units of a stage are dealt round-robin to the wavefronts; a wavefront moves a unit with one
// global_load_lds_dwordx4 (16 B per lane, no registers, LDS image = operand image).  NST - 1 stages are in flight
// while one is consumed: the L2->LDS traffic of this GEMM needs tens of KiB in flight per CU to cover its latency.
// One s_barrier per stage: a wavefront passes it after its own loads of the stage about to be consumed have
// landed (vmcnt) and, having passed it, knows that every wavefront is done with the stage consumed before, which
// is the one the next loads overwrite.
// LDS read of one MFMA operand fragment with a compile-time offset (no address arithmetic in the main loop).
template <int OFF>
__device__ __forceinline__ void lds_read_frag(f16x8 &dst, unsigned base) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(base), "n"(OFF));
}
template <int N, int STRIDE, int KOFF, int I = 0>
__device__ __forceinline__ void lds_read_frags(f16x8 (&dst)[N], unsigned base) {
    if constexpr (I < N) {
        lds_read_frag<I * STRIDE + KOFF>(dst[I], base);
        lds_read_frags<N, STRIDE, KOFF, I + 1>(dst, base);
    }
}

// NWL of the NW wavefronts issue the loads (0 = all of them).  With eight wavefronts (two per SIMD) and NWL = 4 four
// of them issue the loads of all while the other four, which have none to issue, go straight to their MFMAs behind
// the barrier (assuming the usual placement of a workgroup's wavefronts round-robin over the four SIMDs, w and w + 4
// share one; nothing depends on it but the size of the gain): a vector-memory instruction holds up the wavefront that
// issues it, and with all wavefronts issuing at once the matrix unit idles meanwhile (measured on MI355X with
// 256 x 256 tiles: +2-3 % at 8192 tokens, +6 % at 512).
//
// BUF_LOADS issues the loads as buffer loads (one resource descriptor per operand matrix, the unit's offset in a
// scalar register, the lane's 16 bytes as the only vector operand) instead of global loads with a 64-bit address per
// lane: no vector-ALU address arithmetic in the loop and a cheaper address path (256 x 256 tiles: another +2-4 % on top
// of the loading wavefronts; no gain for the 128 x 128 tiles).  Offsets are 32-bit: the host selects such an
// instantiation only for operand matrices below 4 GiB.
template <int FS, int TS, int WF, int WT, int BKT, int NST, int EPI, bool ASM_READS = true, int NWL_ = 0, bool BUF_LOADS = false>
__global__ __launch_bounds__(64 * WF * WT) void gemm_dl_kernel(GemmArgs a) {
    constexpr int NW = WF * WT;
    constexpr int NWL = NWL_ > 0 ? NWL_ : NW;
    constexpr int FW = FS / WF, TW = TS / WT;
    constexpr int NP = FS + TS;
    constexpr int UNITS = NP * BKT;
    static_assert(NWL <= NW && UNITS % NWL == 0, "units must divide evenly over the loading wavefronts");
    static_assert(NST >= 3 && NST <= 6, "ring of 3 or 4 stages (the stage being refilled must differ from the one just published)");
    static_assert(BKT == 2 || BKT == 4, "fragment double-buffer parity needs an even number of k-tiles per stage");
    constexpr int LPW = UNITS / NWL;
    constexpr int STAGE = UNITS * 1024;
    static_assert((NST - 1) * LPW < 64, "vmcnt range");
    static_assert(FW + TW < 16, "lgkmcnt range");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Everything that depends on the wavefront index is kept in scalar registers (readfirstlane makes the index
    // provably uniform): the main loop then spends its vector-ALU slots on MFMAs, not on address arithmetic.  The
    // matrix unit only runs ahead while the wavefront keeps issuing MFMAs, so every VALU instruction between two
    // groups of MFMAs is matrix-unit idle time.
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wf = w % WF, wt = w / WF;
    int nblk = gridDim.x, bid = blockIdx.x;
    // Workgroups are dealt to the XCDs round-robin: give every XCD a contiguous range of tiles, ...
    if (a.n_xcd > 1 && nblk % a.n_xcd == 0) bid = (bid % a.n_xcd) * (nblk / a.n_xcd) + bid / a.n_xcd;
    // ... and walk that range in groups of group_f feature blocks, feature block fastest: the tiles resident on an
    // XCD at one time then form a group_f x (residents / group_f) rectangle, whose operands (group_f weight blocks +
    // the rectangle's token blocks) are fetched into that XCD's L2 once instead of once per tile.
    int tb, fb;
    {
        const int G = a.group_f > 0 ? a.group_f : 1;
        const int per_group = G * a.n_tblk, g = bid / per_group, r = bid - g * per_group;
        const int n_fblk = nblk / a.n_tblk;
        int gf = n_fblk - g * G;
        if (gf > G) gf = G;
        fb = g * G + r % gf, tb = r / gf;
    }
    const int ft0 = fb * FS, tt0 = tb * TS;
    const int z = blockIdx.z;
    const int ktile0 = z * a.ksteps_per_split * 4;  // ksteps_per_split counts 64-wide steps = 4 k-tiles
    int ktiles = (a.Kp >> 4) - ktile0;
    if (ktiles > a.ksteps_per_split * 4) ktiles = a.ksteps_per_split * 4;
    const int nsteps = ktiles / BKT;  // Kp is a multiple of 64 and BKT divides 4

    const size_t strip_bytes = (size_t)(a.Kp >> 4) * 1024;
    const char *ub[LPW];  // this wavefront's units: uniform global address of k-step 0 (lane offset added at the load)
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int u = (w % NWL) + NWL * i, p = u / BKT, kt = u % BKT;
        const char *base;
        if (p < FS) {
            int s = ft0 + p;
            if (s >= a.n_ftiles) s = a.n_ftiles - 1;  // out-of-range strips duplicate a valid one; never stored
            base = (const char *)a.W + (size_t)s * strip_bytes;
        } else {
            int s = tt0 + (p - FS);
            if (s >= a.n_ttiles) s = a.n_ttiles - 1;
            base = (const char *)a.X + (size_t)s * strip_bytes;
        }
        ub[i] = base + (size_t)(ktile0 + kt) * 1024;
    }
    const unsigned lane_off = lane * 16;
#if defined(__HIP_DEVICE_COMPILE__)  // the resource type and the buffer builtins exist in the device pass only
    __amdgpu_buffer_rsrc_t rsrc_w, rsrc_x;
    unsigned uoff[LPW];
    bool uis_w[LPW];
    if constexpr (BUF_LOADS) {
        constexpr int kRawDwords = 0x00020000;  // descriptor word 3: untyped 32-bit data, no swizzle
        rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.W, 0, (unsigned)((size_t)a.n_ftiles * strip_bytes), kRawDwords);
        rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.X, 0, (unsigned)((size_t)a.n_ttiles * strip_bytes), kRawDwords);
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            uis_w[i] = ((w % NWL) + NWL * i) / BKT < FS;
            uoff[i] = (unsigned)(ub[i] - (uis_w[i] ? (const char *)a.W : (const char *)a.X));
        }
    }
#endif
    auto issue = [&](int ks) {
        if (NWL < NW && w >= NWL) return;  // a wavefront that loads nothing has nothing outstanding: its vmcnt waits fall through
        char *dst = smem + (ks % NST) * STAGE + w * 1024;
#if defined(__HIP_DEVICE_COMPILE__)
        if constexpr (BUF_LOADS) {
            const unsigned kbytes = (unsigned)ks * (BKT * 1024);
#pragma unroll
            for (int i = 0; i < LPW; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(uis_w[i] ? rsrc_w : rsrc_x, (__attribute__((address_space(3))) void *)(dst + i * (NWL * 1024)), 16,
                                                         (int)lane_off, (int)(uoff[i] + kbytes), 0, 0);
            return;
        }
#endif
        const size_t koff = (size_t)ks * (BKT * 1024);
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ub[i] + koff + lane_off),
                                             (__attribute__((address_space(3))) void *)(dst + i * (NWL * 1024)), 16, 0, 0);
    };

    auto issue_unit = [&](int ks, int i) {  // unit i of this wavefront's share of step ks (i is a constant after unrolling)
        char *dst = smem + (ks % NST) * STAGE + w * 1024 + i * (NWL * 1024);
#if defined(__HIP_DEVICE_COMPILE__)
        if constexpr (BUF_LOADS) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(uis_w[i] ? rsrc_w : rsrc_x, (__attribute__((address_space(3))) void *)dst, 16, (int)lane_off,
                                                     (int)(uoff[i] + (unsigned)ks * (BKT * 1024)), 0, 0);
            return;
        }
#endif
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ub[i] + (size_t)ks * (BKT * 1024) + lane_off),
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };

    f32x16 acc[FW][TW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    // what follows the k loop: the row-major epilogues go through LDS (every wavefront is done with the operand
    // stages once the workgroup has passed the barrier), the tile-ordered one stores as it stands
    auto finish = [&]() {
        if constexpr (EPI != EPI_SWIGLU) {
            static_assert(NW * kEpiScratch <= NST * STAGE, "the epilogue scratch lives in the operand ring");
            __syncthreads();
            gemm_epilogue_rows<FW, TW, EPI>(a, acc, ft0 + wf * FW, tt0 + wt * TW, z, lane, smem + w * kEpiScratch);
        } else {
            gemm_epilogue<FW, TW, EPI>(a, acc, ft0 + wf * FW, tt0 + wt * TW, z, lane);
        }
    };

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < nsteps) issue(s);

    // Software pipeline: operand fragments are read from LDS one k-tile ahead of the MFMAs that use them, also
    // across the stage boundary, so the matrix unit never waits on LDS latency.  The barrier that publishes stage
    // ks + 1 therefore sits before the LAST k-tile of stage ks.
    //
    // The LDS reads are issued with inline assembly and waited for by hand.  Left to the compiler, the wait before
    // each group of MFMAs becomes lgkmcnt(0) wherever control flow merges (loop entry, the branch around the tail
    // prefetch), which also waits for the reads that were issued one instruction earlier and stalls the matrix
    // unit for a full LDS latency per k-tile.  The hand-placed wait is lgkmcnt(FW + TW): LDS reads return in
    // order, so "at most the FW + TW newest outstanding" means the previous group has landed.  (A scalar load in
    // flight can only make that wait more conservative.)
    //
    // The price: between such a read and its wait the compiler believes the destination registers already hold
    // the data, so a register copy or reuse it chose to insert there would be silently wrong.  Every
    // ASM_READS = true instantiation that the library launches is therefore covered by the bit-level parity
    // tests; ASM_READS = false keeps the reads visible to the compiler (always correct, one exposed LDS latency
    // per stage) and is what rarely used instantiations take.
    f16x8 fa[2][FW], fb_[2][TW];
    const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) char *)smem + (wf * FW) * (BKT * 1024) + lane * 16;
    const unsigned lds_x = (unsigned)(size_t)(__attribute__((address_space(3))) char *)smem + (FS + wt * TW) * (BKT * 1024) + lane * 16;
    auto read_frags = [&](int buf, int ks, auto kt_tag) {
        constexpr int KT = decltype(kt_tag)::value;
        const unsigned so = (ks % NST) * STAGE;
        if constexpr (ASM_READS) {
            const unsigned bw = lds_w + so, bx = lds_x + so;
            if (buf == 0) {
                lds_read_frags<FW, BKT * 1024, KT * 1024>(fa[0], bw);
                lds_read_frags<TW, BKT * 1024, KT * 1024>(fb_[0], bx);
            } else {
                lds_read_frags<FW, BKT * 1024, KT * 1024>(fa[1], bw);
                lds_read_frags<TW, BKT * 1024, KT * 1024>(fb_[1], bx);
            }
        } else {
            const char *bw = smem + (wf * FW) * (BKT * 1024) + lane * 16 + so;
            const char *bx = smem + (FS + wt * TW) * (BKT * 1024) + lane * 16 + so;
#pragma unroll
            for (int i = 0; i < FW; ++i) fa[buf][i] = *(const f16x8 *)(bw + (i * BKT + KT) * 1024);
#pragma unroll
            for (int j = 0; j < TW; ++j) fb_[buf][j] = *(const f16x8 *)(bx + (j * BKT + KT) * 1024);
            __builtin_amdgcn_sched_barrier(0);  // issued here, ahead of the MFMAs that hide their latency
        }
    };
    auto frags_ready = [&](int buf, bool newer_in_flight) {
        if constexpr (ASM_READS) {
            if (newer_in_flight) wait_lgkmcnt<FW + TW>();
            else wait_lgkmcnt<0>();
            // tie the registers to the wait: the MFMAs below must not be scheduled above it
#pragma unroll
            for (int i = 0; i < FW; ++i) asm volatile("" : "+v"(fa[buf][i]));
#pragma unroll
            for (int j = 0; j < TW; ++j) asm volatile("" : "+v"(fb_[buf][j]));
        }
    };
    auto publish_next = [&](int ks) {
        // loads issued after those of step ks + 1 (and still allowed in flight): steps ks + 2 .. ks + NST - 2
        const int later = nsteps - 2 - ks;
        if (NST >= 4 && later >= NST - 3) wait_vmcnt<(NST >= 4 ? NST - 3 : 0) * LPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (ks + NST - 1 < nsteps) issue(ks + NST - 1);
    };
    if (nsteps > 0) {
        wait_vmcnt<0>();  // prologue: stage 0 (whatever else is in flight lands too; once per kernel)
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, std::integral_constant<int, 0>{});
    }
    auto mfma_group = [&](int c) {
#pragma unroll
        for (int i = 0; i < FW; ++i)
#pragma unroll
            for (int j = 0; j < TW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[c][i], fb_[c][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);  // later waits and barriers stay behind these MFMAs
    };
    // ---- interleaved pipeline (stages of two k-tiles, hand-issued LDS reads) ----------------------------------------
    // Nothing is issued in bursts: inside the group of MFMAs of one k-tile, the LDS read of one operand fragment of the
    // NEXT k-tile follows each of the first FW + TW MFMAs, and a loading wavefront also drops its global->LDS loads
    // between the MFMAs, evenly spaced -- the first half of a step's loads in the group behind the barrier that frees
    // their ring slot, the second half in the group after it.  Measured on MI355X against issuing the FW + TW reads
    // ahead of the group and all loads right behind the barrier (256 x 256 tiles, K = 4096): 1.29 -> 1.41 PFLOP/s at
    // 8192 tokens, 1.04 -> 1.23 at 512: with every wavefront of the workgroup released by the same barrier, bursts of
    // LDS and vector-memory instructions queue up in front of the MFMAs of the wavefronts that issued them.
    // The operands of a group are waited for with lgkmcnt(0) right behind the group that issued their reads; the last of
    // them was issued two MFMAs (and the other wavefront's share of the SIMD) before.  The loop is cut into regions so
    // that "this group carries loads" is a compile-time property and each region's body is straight-line code; a
    // wavefront that loads nothing runs the same regions without loads.
    if constexpr (BKT == 2 && ASM_READS && FW + TW <= FW * TW) {
        auto group = [&](auto cur_tag, int ks_next, auto kt_tag, auto l0_tag, auto l1_tag, int ks_load) {
            constexpr int CUR = decltype(cur_tag)::value, NXT = 1 - CUR, KT = decltype(kt_tag)::value, M = FW * TW, R = FW + TW;
            constexpr int L0 = decltype(l0_tag)::value, NL = decltype(l1_tag)::value - L0;
            const unsigned so = (ks_next % NST) * STAGE;
            const unsigned bw = lds_w + so, bx = lds_x + so;
            auto step = [&](auto self, auto m_tag) {
                constexpr int MI = decltype(m_tag)::value;
                acc[MI / TW][MI % TW] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[CUR][MI / TW], fb_[CUR][MI % TW], acc[MI / TW][MI % TW], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);  // the order written here is the order issued
                if constexpr (KT >= 0 && MI < R) {
                    if constexpr (MI < FW) lds_read_frag<(MI * BKT + (KT >= 0 ? KT : 0)) * 1024>(fa[NXT][MI], bw);
                    else lds_read_frag<((MI - FW) * BKT + (KT >= 0 ? KT : 0)) * 1024>(fb_[NXT][MI - FW], bx);
                }
                if constexpr (NL > 0)
                    if constexpr (((MI + 1) * NL) / M != (MI * NL) / M) issue_unit(ks_load, L0 + (MI * NL) / M);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (MI + 1 < M) self(self, std::integral_constant<int, MI + 1>{});
            };
            step(step, std::integral_constant<int, 0>{});
        };
        auto landed = [&](int buf) {  // every LDS read issued so far has returned; ties the registers to the wait
            wait_lgkmcnt<0>();
#pragma unroll
            for (int i = 0; i < FW; ++i) asm volatile("" : "+v"(fa[buf][i]));
#pragma unroll
            for (int j = 0; j < TW; ++j) asm volatile("" : "+v"(fb_[buf][j]));
        };
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using NoRead = std::integral_constant<int, -1>;
        using LHalf = std::integral_constant<int, (LPW + 1) / 2>;
        using LAll = std::integral_constant<int, LPW>;
        const int n_load_steps = nsteps - (NST - 1);  // steps whose barrier also frees the slot of a step still to be loaded
        // LA: the first group issues the second half of the loads that the previous stage's barrier released;
        // LB: the group behind this stage's barrier issues the first half of the loads of step ks + NST - 1.
        auto stage2 = [&](int ks, auto has_next, auto la_tag, auto lb_tag) {
            constexpr bool LA = decltype(la_tag)::value, LB = decltype(lb_tag)::value;
            if constexpr (LA) group(I0{}, ks, I1{}, LHalf{}, LAll{}, ks - 1 + NST - 1);
            else group(I0{}, ks, I1{}, I0{}, I0{}, 0);
            landed(1);
            if constexpr (decltype(has_next)::value) {
                // own loads of step ks + 1 landed: at most those of the NST - 3 newer steps stay in flight
                if constexpr (LB) {
                    wait_vmcnt<(NST >= 4 ? NST - 3 : 0) * LPW>();
                } else {
                    const int later = nsteps - 2 - ks;
                    if (NST >= 4 && later >= NST - 3) wait_vmcnt<(NST >= 4 ? NST - 3 : 0) * LPW>();
                    else wait_vmcnt<0>();
                }
                __builtin_amdgcn_s_barrier();  // step ks + 1 visible to all; every wavefront is done with step ks - 1
                if constexpr (LB) group(I1{}, ks + 1, I0{}, I0{}, LHalf{}, ks + NST - 1);
                else group(I1{}, ks + 1, I0{}, I0{}, I0{}, 0);
                landed(0);  // see below: no hand-issued read is in flight when a stage ends
            } else {
                group(I1{}, 0, NoRead{}, I0{}, I0{}, 0);
            }
        };
        auto run = [&](auto loader_tag) {
            using T_ = std::true_type;
            using F_ = std::false_type;
            using L_ = std::integral_constant<bool, decltype(loader_tag)::value>;
            int ks = 0;
            if (n_load_steps >= 1) {
                stage2(0, T_{}, F_{}, L_{});
                for (ks = 1; ks < n_load_steps; ++ks) stage2(ks, T_{}, L_{}, L_{});
                stage2(ks, T_{}, L_{}, F_{});  // NST >= 3: a next step exists
                ++ks;
            }
            for (; ks + 1 < nsteps; ++ks) stage2(ks, T_{}, F_{}, F_{});
            stage2(nsteps - 1, F_{}, F_{}, F_{});
        };
        // A hand-issued read is invisible to the compiler: until the wait, it takes the destination registers for
        // valid and may copy them, which it does wherever two code regions disagree on the register assignment (the
        // edges between the regions below, a loop's back edge).  So no such read is ever in flight across an edge:
        // every stage, and the prologue's read of the first k-tile, ends with the wait for what it issued.  Inside a
        // stage the code between a read and its wait is straight-line.
        if (nsteps > 0) {
            landed(0);
            if (NWL == NW || w < NWL) run(std::true_type{});
            else run(std::false_type{});
        }
        finish();
        return;
    }
    // ---- generic pipeline (four k-tiles per stage, or compiler-visible LDS reads) ----------------------------------------
    // One stage of MFMAs.  HAS_NEXT is a compile-time flag so that the steady-state loop body is straight-line code.
    auto stage = [&](int ks, auto has_next) {
        // k-tiles 0 .. BKT-2: prefetch the next k-tile of this stage, then multiply the current one
        read_frags(1, ks, std::integral_constant<int, 1>{});
        frags_ready(0, true);
        mfma_group(0);
        if constexpr (BKT == 4) {
            read_frags(0, ks, std::integral_constant<int, 2>{});
            frags_ready(1, true);
            mfma_group(1);
            read_frags(1, ks, std::integral_constant<int, 3>{});
            frags_ready(0, true);
            mfma_group(0);
        }
        // last k-tile: publish the next stage and prefetch its first k-tile, so that the MFMAs of this k-tile
        // (operands read long before) run right behind the barrier and cover the LDS latency of the prefetch.
        // (Placing the barrier in the middle of this k-tile's MFMAs instead measured about 3% slower.)
        if constexpr (decltype(has_next)::value) {
            publish_next(ks);
            read_frags(0, ks + 1, std::integral_constant<int, 0>{});
            frags_ready(1, true);
        } else {
            frags_ready(1, false);
        }
        mfma_group(1);
    };
    for (int ks = 0; ks + 1 < nsteps; ++ks) stage(ks, std::true_type{});
    if (nsteps > 0) stage(nsteps - 1, std::false_type{});
    finish();
}

// ---- weight-streaming GEMM of a decode batch -------------------------------------------------------------------
// With at most 128 tokens every weight byte is used once (by up to four MFMAs), so the GEMM is a sweep over the
// weights (Sec. 2.3: decode is bound by memory traffic) and its speed on a share of the chip is set by the bytes
// each CU keeps in flight:
// one CU draws at most about 50 GB/s from HBM and needs on the order of 100 KiB outstanding to get there.  An LDS
// ring cannot hold that much beside its resident stages, and nothing here is shared between wavefronts anyway:
// each wavefront owns FW feature strips and all tokens.  So the weights bypass LDS: the P32 tile order makes a
// 1 KiB tile exactly one MFMA A-operand, fetched by one 16-byte-per-lane load straight into registers, DST stages
// (DST * BKT tiles per strip) ahead of use.  Only the activations, which every wavefront of the workgroup needs,
// go through a small asynchronous LDS ring of NSX = DST + 1 stages.
//
// Per-element summation order (k-tiles in sequence, slices of the k range in the partial buffer) is the same as
// in gemm_dl_kernel, so the two are interchangeable bit for bit.
template <int FW, int TW, int NW, int BKT, int DST, int EPI>
__global__ __launch_bounds__(64 * NW) void gemm_stream_kernel(GemmArgs a) {
    constexpr int NSX = DST + 1;
    constexpr int XUNITS = TW * BKT;  // 1 KiB activation tiles per stage
    static_assert(XUNITS % NW == 0, "activation tiles must divide evenly over the wavefronts");
    constexpr int LPWX = XUNITS / NW;
    constexpr int XSTAGE = XUNITS * 1024;
    constexpr int PER_STAGE = LPWX + BKT * FW;  // vector-memory instructions a wavefront issues per stage
    static_assert((DST - 1) * PER_STAGE < 64, "vmcnt range");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tb = blockIdx.x % a.n_tblk, fb = blockIdx.x / a.n_tblk;
    const int ft0 = (fb * NW + w) * FW, tt0 = tb * TW;
    const int z = blockIdx.z;
    const int ktile0 = z * a.ksteps_per_split * 4;
    int ktiles = (a.Kp >> 4) - ktile0;
    if (ktiles > a.ksteps_per_split * 4) ktiles = a.ksteps_per_split * 4;
    const int nsteps = ktiles / BKT;  // >= DST: the host launches this kernel only then

    const size_t strip_bytes = (size_t)(a.Kp >> 4) * 1024;
    const unsigned lane_off = lane * 16;
    const char *wb[FW];  // uniform: k-step 0 of this wavefront's weight strips
#pragma unroll
    for (int i = 0; i < FW; ++i) {
        int s = ft0 + i;
        if (s >= a.n_ftiles) s = a.n_ftiles - 1;  // out-of-range strips duplicate a valid one; never stored
        wb[i] = (const char *)a.W + (size_t)s * strip_bytes + (size_t)ktile0 * 1024;
    }
    const char *xb[LPWX];  // uniform: k-step 0 of the activation tiles this wavefront fetches
#pragma unroll
    for (int i = 0; i < LPWX; ++i) {
        const int u = w + NW * i, ts = u / BKT, kt = u % BKT;
        int s = tt0 + ts;
        if (s >= a.n_ttiles) s = a.n_ttiles - 1;
        xb[i] = (const char *)a.X + (size_t)s * strip_bytes + (size_t)(ktile0 + kt) * 1024;
    }
    auto issue_x = [&](int ks) {
        char *dst = smem + (ks % NSX) * XSTAGE + w * 1024;
        const size_t koff = (size_t)ks * (BKT * 1024);
#pragma unroll
        for (int i = 0; i < LPWX; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(xb[i] + koff + lane_off),
                                             (__attribute__((address_space(3))) void *)(dst + i * (NW * 1024)), 16, 0, 0);
    };
    // Weight loads are ordinary loads: the compiler knows when their registers are valid (an inline-assembly load
    // would return into registers the compiler is free to copy or reuse before the data lands).  It may move them
    // within a stage, never across the stage barriers, which is all the counted waits below rely on.
    f16x8 wr[DST][FW][BKT];
    auto issue_w = [&](auto d_tag, int ks) {
        constexpr int D = decltype(d_tag)::value;
        const size_t koff = (size_t)ks * (BKT * 1024) + lane_off;
#pragma unroll
        for (int i = 0; i < FW; ++i)
#pragma unroll
            for (int kt = 0; kt < BKT; ++kt)  // every weight byte is used once: streaming (non-temporal) loads leave the caches to the other phase
                wr[D][i][kt] = __builtin_nontemporal_load((const f16x8 *)(wb[i] + koff + kt * 1024));
    };

    f32x16 acc[FW][TW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // One stage.  D = register set (stage index modulo DST), PREFETCH = whether stage ks + DST exists; both are
    // compile-time so that the loop bodies below are straight-line code and the waits stay exact.  Loads complete
    // in issue order and the load sets of different stages are separated by barriers: when at most the loads of
    // the DST - 1 newer stages are outstanding, everything of stage ks has landed.
    auto stage = [&](auto d_tag, auto prefetch_tag, int ks, int newer_stages) {
        constexpr int D = decltype(d_tag)::value;
        // own activation tiles of stage ks landed: at most the loads of the DST - 1 newer stages stay in flight
        if (newer_stages >= DST - 1) wait_vmcnt<(DST - 1) * PER_STAGE>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();  // stage ks visible to all; every wavefront is done with stage ks - 1
        if constexpr (decltype(prefetch_tag)::value) issue_x(ks + DST);  // into the slot of stage ks - 1
        const char *xs = smem + (ks % NSX) * XSTAGE + lane_off;
#pragma unroll
        for (int kt = 0; kt < BKT; ++kt) {
            f16x8 xf[TW];
#pragma unroll
            for (int j = 0; j < TW; ++j) xf[j] = *(const f16x8 *)(xs + (j * BKT + kt) * 1024);
#pragma unroll
            for (int i = 0; i < FW; ++i)
#pragma unroll
                for (int j = 0; j < TW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wr[D][i][kt], xf[j], acc[i][j], 0, 0, 0);
        }
        if constexpr (decltype(prefetch_tag)::value) issue_w(d_tag, ks + DST);
    };
    // group of N consecutive stages starting at a multiple of DST; the first PF of them prefetch
    auto group = [&](auto n_tag, auto pf_tag, int s0) {
        constexpr int N = decltype(n_tag)::value, PF = decltype(pf_tag)::value;
        auto one = [&](auto i_tag) {
            constexpr int I = decltype(i_tag)::value;
            if constexpr (I < N) {
                stage(std::integral_constant<int, I % DST>{}, std::integral_constant<bool, (I < PF)>{}, s0 + I,
                      PF == N ? DST - 1 : (N - 1 - I));
            }
        };
        one(std::integral_constant<int, 0>{});
        one(std::integral_constant<int, 1>{});
        one(std::integral_constant<int, 2>{});
        one(std::integral_constant<int, 3>{});
        one(std::integral_constant<int, 4>{});
        one(std::integral_constant<int, 5>{});
        one(std::integral_constant<int, 6>{});
        one(std::integral_constant<int, 7>{});
    };
    static_assert(2 * DST <= 8, "group() unrolls at most 8 stages");

    // prologue: stages 0 .. DST-1 in flight (activation tiles first within each stage, as in the steady state)
    {
        auto pro = [&](auto d_tag) {
            constexpr int D = decltype(d_tag)::value;
            if constexpr (D < DST) {
                issue_x(D);
                issue_w(d_tag, D);
                __builtin_amdgcn_sched_barrier(0);  // keep the stages' load sets in order (no barrier between them here)
            }
        };
        pro(std::integral_constant<int, 0>{});
        pro(std::integral_constant<int, 1>{});
        pro(std::integral_constant<int, 2>{});
        pro(std::integral_constant<int, 3>{});
    }
    static_assert(DST <= 4, "prologue unrolls at most 4 stages");
    int s0 = 0;
    for (; s0 + 2 * DST <= nsteps; s0 += DST) group(std::integral_constant<int, DST>{}, std::integral_constant<int, DST>{}, s0);
    // DST + r stages remain (0 <= r < DST): the first r still prefetch
    const int r = nsteps - s0 - DST;
    if (r == 0) group(std::integral_constant<int, DST>{}, std::integral_constant<int, 0>{}, s0);
    if constexpr (DST >= 2) if (r == 1) group(std::integral_constant<int, DST + 1>{}, std::integral_constant<int, 1>{}, s0);
    if constexpr (DST >= 3) if (r == 2) group(std::integral_constant<int, DST + 2>{}, std::integral_constant<int, 2>{}, s0);
    if constexpr (DST >= 4) if (r == 3) group(std::integral_constant<int, DST + 3>{}, std::integral_constant<int, 3>{}, s0);
    gemm_epilogue<FW, TW, EPI>(a, acc, ft0, tt0, z, lane);
}

// Finishes a split-K GEMM: sums the S fp32 partials in slice order and applies the epilogue.
// One thread per (token, 4 consecutive packed rows).
struct ReduceArgs {
    const float *partial;  // [S][T][N]
    int S, T, N;
    void *out;
    const void *res;
    const bf16_t *bias;
    int ld_out;
    f16_t *out_p32;
    int out_Kp;
};

template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(ReduceArgs a) {
    const int quads = a.N >> 2;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)a.T * quads) return;
    const int t = (int)(idx / quads), n = (int)(idx % quads) * 4;
    if constexpr (EPI == EPI_SWIGLU) {
        // packed rows: strip s holds gate features [16s, 16s+16) in rows 0..15, the matching up features in 16..31
        const int strip = n >> 5;
        if (n & 16) return;
        float gsum[4], usum[4];
        sum_slices4(a.partial + (size_t)t * a.N + n, (size_t)a.T * a.N, a.S, gsum);
        sum_slices4(a.partial + (size_t)t * a.N + n + 16, (size_t)a.T * a.N, a.S, usum);
        const int f = strip * 16 + (n & 15);
        uint2 o = {packh2(silu_f(gsum[0]) * usum[0], silu_f(gsum[1]) * usum[1]),
                   packh2(silu_f(gsum[2]) * usum[2], silu_f(gsum[3]) * usum[3])};
        *(uint2 *)(a.out_p32 + p32_offset(t, f, a.out_Kp)) = o;
    } else {
        float v[4];
        sum_slices4(a.partial + (size_t)t * a.N + n, (size_t)a.T * a.N, a.S, v);
        if constexpr (EPI == EPI_ROWMAJOR) {
            if (a.bias) {
                uint2 bb = *(const uint2 *)(a.bias + n);
                v[0] += bf2f(bb.x & 0xffff), v[1] += bf2f(bb.x >> 16), v[2] += bf2f(bb.y & 0xffff), v[3] += bf2f(bb.y >> 16);
            }
            uint2 o = {packh2(v[0], v[1]), packh2(v[2], v[3])};
            *(uint2 *)((f16_t *)a.out + (size_t)t * a.ld_out + n) = o;
        } else if constexpr (EPI == EPI_RES_IN) {
            uint2 rr = *(const uint2 *)((const bf16_t *)a.res + (size_t)t * a.ld_out + n);
            float4 o = {v[0] + bf2f(rr.x & 0xffff), v[1] + bf2f(rr.x >> 16), v[2] + bf2f(rr.y & 0xffff), v[3] + bf2f(rr.y >> 16)};
            *(float4 *)((float *)a.out + (size_t)t * a.ld_out + n) = o;
        } else {
            float4 rr = *(const float4 *)((const float *)a.res + (size_t)t * a.ld_out + n);
            uint2 o = {pack2(v[0] + rr.x, v[1] + rr.y), pack2(v[2] + rr.z, v[3] + rr.w)};
            *(uint2 *)((bf16_t *)a.out + (size_t)t * a.ld_out + n) = o;
        }
    }
}

}  // namespace nexus
