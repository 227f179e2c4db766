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
    EPI_SWIGLU = 2,    // weight strips alternate gate/up; out_p32[t][f] = half(silu(gate) * up)
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
#pragma unroll
            for (int i = 0; i < FW; i += 2) {
                const int ft = ft0 + i;
                if (ft >= a.n_ftiles) continue;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int f = (ft >> 1) * 32 + 8 * b + 4 * g;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = silu_f(acc[i][j][4 * b + e]) * acc[i + 1][j][4 * b + e];
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

// s_waitcnt on the vector-memory counter alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters
// left at their maxima).  Asynchronous global->LDS loads are tracked by this counter.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// ---- main GEMM: asynchronous global->LDS tile loads, NST-stage ring --------------------------------------------
// A stage holds BKT k-tiles (16 k each) of FS weight strips and TS token strips, as 1 KiB units in P32 order.
// The units of a stage are dealt round-robin to the wavefronts; a wavefront moves a unit with one
// global_load_lds_dwordx4 (16 B per lane, no registers, LDS image = operand image).  NST - 1 stages are in flight
// while one is consumed: the L2->LDS traffic of this GEMM needs tens of KiB in flight per CU to cover its latency.
// One s_barrier per stage: a wavefront passes it after its own loads of the stage about to be consumed have
// landed (vmcnt) and, having passed it, knows that every wavefront is done with the stage consumed before, which
// is the one the next loads overwrite.
template <int FS, int TS, int WF, int WT, int BKT, int NST, int EPI>
__global__ __launch_bounds__(64 * WF * WT) void gemm_dl_kernel(GemmArgs a) {
    constexpr int NW = WF * WT;
    constexpr int FW = FS / WF, TW = TS / WT;
    constexpr int NP = FS + TS;
    constexpr int UNITS = NP * BKT;
    static_assert(UNITS % NW == 0, "units must divide evenly over the wavefronts");
    static_assert(EPI != EPI_SWIGLU || FW % 2 == 0, "gate/up strip pairs stay in one wavefront");
    static_assert(NST >= 3 && NST <= 4, "ring of 3 or 4 stages (the stage being refilled must differ from the one just published)");
    static_assert(BKT == 2 || BKT == 4, "fragment double-buffer parity needs an even number of k-tiles per stage");
    constexpr int LPW = UNITS / NW;
    constexpr int STAGE = UNITS * 1024;
    static_assert((NST - 1) * LPW < 64, "vmcnt range");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wf = w % WF, wt = w / WF;
    int nblk = gridDim.x, bid = blockIdx.x;
    if (a.n_xcd > 1 && nblk % a.n_xcd == 0) bid = (bid % a.n_xcd) * (nblk / a.n_xcd) + bid / a.n_xcd;
    const int tb = bid % a.n_tblk, fb = bid / a.n_tblk;
    const int ft0 = fb * FS, tt0 = tb * TS;
    const int z = blockIdx.z;
    const int ktile0 = z * a.ksteps_per_split * 4;  // ksteps_per_split counts 64-wide steps = 4 k-tiles
    int ktiles = (a.Kp >> 4) - ktile0;
    if (ktiles > a.ksteps_per_split * 4) ktiles = a.ksteps_per_split * 4;
    const int nsteps = ktiles / BKT;  // Kp is a multiple of 64 and BKT divides 4

    const size_t strip_bytes = (size_t)(a.Kp >> 4) * 1024;
    const char *ub[LPW];  // this wavefront's units: global address of k-step 0, this lane
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int u = w + NW * i, p = u / BKT, kt = u % BKT;
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
        ub[i] = base + (size_t)(ktile0 + kt) * 1024 + lane * 16;
    }
    auto issue = [&](int ks) {
        char *dst = smem + (ks % NST) * STAGE + w * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ub[i] + (size_t)ks * (BKT * 1024)),
                                             (__attribute__((address_space(3))) void *)(dst + i * (NW * 1024)), 16, 0, 0);
    };

    f32x16 acc[FW][TW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < nsteps) issue(s);

    // Software pipeline: operand fragments are read from LDS one k-tile ahead of the MFMAs that use them, also
    // across the stage boundary, so the matrix unit never waits on LDS latency.  The barrier that publishes stage
    // ks + 1 therefore sits before the LAST k-tile of stage ks.
    f16x8 fa[2][FW], fb_[2][TW];
    auto read_frags = [&](int buf, int ks, int kt) {
        const char *sW = smem + (ks % NST) * STAGE + (wf * FW) * (BKT * 1024) + kt * 1024 + lane * 16;
        const char *sX = smem + (ks % NST) * STAGE + (FS + wt * TW) * (BKT * 1024) + kt * 1024 + lane * 16;
#pragma unroll
        for (int i = 0; i < FW; ++i) fa[buf][i] = *(const f16x8 *)(sW + i * (BKT * 1024));
#pragma unroll
        for (int j = 0; j < TW; ++j) fb_[buf][j] = *(const f16x8 *)(sX + j * (BKT * 1024));
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
        read_frags(0, 0, 0);
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): enter the loop with nothing pending (see the loop's end)
    }
    // One stage of MFMAs.  HAS_NEXT is a compile-time flag so that the steady-state loop body is straight-line
    // code: with a branch around the next stage's fragment reads, the two paths would merge with different
    // numbers of LDS reads pending and the compiler would have to wait for all of them before the MFMAs.
    auto stage = [&](int ks, auto has_next) {
#pragma unroll
        for (int kt = 0; kt < BKT; ++kt) {
            const int c = kt & 1;
            if (kt == BKT - 1) {
                if constexpr (decltype(has_next)::value) {
                    publish_next(ks);
                    read_frags(c ^ 1, ks + 1, 0);
                }
            } else {
                read_frags(c ^ 1, ks, kt + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < FW; ++i)
#pragma unroll
                for (int j = 0; j < TW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[c][i], fb_[c][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // The fragments of the next stage's first k-tile were requested a whole k-tile of MFMAs ago: settle the
        // LDS counter here, at no cost, so that no read is pending across the loop back-edge (where the compiler
        // would otherwise wait for everything, including the reads it has just issued).
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    };
    for (int ks = 0; ks + 1 < nsteps; ++ks) stage(ks, std::true_type{});
    if (nsteps > 0) stage(nsteps - 1, std::false_type{});
    gemm_epilogue<FW, TW, EPI>(a, acc, ft0 + wf * FW, tt0 + wt * TW, z, lane);
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
        // packed rows: strip 2s holds gate features [32s, 32s+32), strip 2s+1 the matching up features
        const int strip = n >> 5;
        if (strip & 1) return;
        float gsum[4] = {0, 0, 0, 0}, usum[4] = {0, 0, 0, 0};
        for (int s = 0; s < a.S; ++s) {
            const float *p = a.partial + ((size_t)s * a.T + t) * a.N + n;
            float4 gv = *(const float4 *)p, uv = *(const float4 *)(p + 32);
            gsum[0] += gv.x, gsum[1] += gv.y, gsum[2] += gv.z, gsum[3] += gv.w;
            usum[0] += uv.x, usum[1] += uv.y, usum[2] += uv.z, usum[3] += uv.w;
        }
        const int f = (strip >> 1) * 32 + (n & 31);
        uint2 o = {packh2(silu_f(gsum[0]) * usum[0], silu_f(gsum[1]) * usum[1]),
                   packh2(silu_f(gsum[2]) * usum[2], silu_f(gsum[3]) * usum[3])};
        *(uint2 *)(a.out_p32 + p32_offset(t, f, a.out_Kp)) = o;
    } else {
        float v[4] = {0, 0, 0, 0};
        for (int s = 0; s < a.S; ++s) {
            float4 pv = *(const float4 *)(a.partial + ((size_t)s * a.T + t) * a.N + n);
            v[0] += pv.x, v[1] += pv.y, v[2] += pv.z, v[3] += pv.w;
        }
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
