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
    if (a.n_xcd > 1 && nblk % a.n_xcd == 0) bid = (bid % a.n_xcd) * (nblk / a.n_xcd) + bid / a.n_xcd;
    const int tb = bid % a.n_tblk, fb = bid / a.n_tblk;
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
        ub[i] = base + (size_t)(ktile0 + kt) * 1024;
    }
    const unsigned lane_off = lane * 16;
    auto issue = [&](int ks) {
        char *dst = smem + (ks % NST) * STAGE + w * 1024;
        const size_t koff = (size_t)ks * (BKT * 1024);
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ub[i] + koff + lane_off),
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
    //
    // The LDS reads are issued with inline assembly and waited for by hand.  Left to the compiler, the wait before
    // each group of MFMAs becomes lgkmcnt(0) wherever control flow merges (loop entry, the branch around the tail
    // prefetch), which also waits for the reads that were issued one instruction earlier and stalls the matrix
    // unit for a full LDS latency per k-tile.  The hand-placed wait is lgkmcnt(FW + TW): LDS reads return in
    // order, so "at most the FW + TW newest outstanding" means the previous group has landed.  (A scalar load in
    // flight can only make that wait more conservative.)
    f16x8 fa[2][FW], fb_[2][TW];
    const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) char *)smem + (wf * FW) * (BKT * 1024) + lane * 16;
    const unsigned lds_x = (unsigned)(size_t)(__attribute__((address_space(3))) char *)smem + (FS + wt * TW) * (BKT * 1024) + lane * 16;
    auto read_frags = [&](int buf, int ks, auto kt_tag) {
        constexpr int KT = decltype(kt_tag)::value;
        const unsigned so = (ks % NST) * STAGE;
        const unsigned bw = lds_w + so, bx = lds_x + so;
        if (buf == 0) {
            lds_read_frags<FW, BKT * 1024, KT * 1024>(fa[0], bw);
            lds_read_frags<TW, BKT * 1024, KT * 1024>(fb_[0], bx);
        } else {
            lds_read_frags<FW, BKT * 1024, KT * 1024>(fa[1], bw);
            lds_read_frags<TW, BKT * 1024, KT * 1024>(fb_[1], bx);
        }
    };
    auto frags_ready = [&](int buf, bool newer_in_flight) {
        if (newer_in_flight) wait_lgkmcnt<FW + TW>();
        else wait_lgkmcnt<0>();
        // tie the registers to the wait: the MFMAs below must not be scheduled above it
#pragma unroll
        for (int i = 0; i < FW; ++i) asm volatile("" : "+v"(fa[buf][i]));
#pragma unroll
        for (int j = 0; j < TW; ++j) asm volatile("" : "+v"(fb_[buf][j]));
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
    };
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
        // last k-tile: publish the next stage and prefetch its first k-tile
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
    gemm_epilogue<FW, TW, EPI>(a, acc, ft0 + wf * FW, tt0 + wt * TW, z, lane);
}

// ---- wide-N GEMM of a prefill chunk: whole-chunk token tile, asymmetric rings ------------------------------------
// A prefill chunk of a few hundred tokens makes the projection GEMMs stream their weights from HBM at a rate close
// to the HBM roofline (arithmetic intensity = chunk length flop/byte), so what limits them is how far ahead of
// use the weight loads can be issued: lookahead = LDS bytes devoted to in-flight weights / consumption rate.  The
// activations of the chunk, by contrast, are a few MiB that every workgroup re-reads from L2.  This kernel
// therefore gives a workgroup ALL token strips of a 512-token block (so weights are fetched once, not once per
// token block) and splits LDS into a deep ring for the small weight stages (NSW stages of FS x BKT KiB) and a
// shallow ring for the large activation stages (NSX stages of 16 x BKT KiB).  Loads are counted per wavefront
// and complete in order, so the two rings are filled by different wavefronts: 0..3 load activations, 4..7 load
// weights; each waits only for its own loads and the stage barrier publishes both.
// Eight wavefronts: wavefront w owns token strips 2w, 2w+1 and all FS feature strips (FS x 2 MFMA tiles).
template <int FS, int BKT, int NSW, int NSX, int EPI>
__global__ __launch_bounds__(512) void gemm_ft_kernel(GemmArgs a) {
    constexpr int TS = 16, FW = FS, TW = 2, NW = 8;
    constexpr int WSTAGE = FS * BKT * 1024, XSTAGE = TS * BKT * 1024;
    constexpr int XLPW = TS * BKT / 4, WLPW = FS * BKT / 4;  // loads per loading wavefront per stage
    static_assert(BKT == 2, "fragment double-buffer parity");
    static_assert((FS * BKT) % 4 == 0, "weight units divide over four wavefronts");
    static_assert(NSX >= 3 && NSW >= 3 && NSW <= 8, "ring depths");
    static_assert(EPI != EPI_SWIGLU || FW % 2 == 0, "gate/up strip pairs stay in one wavefront");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *ringW = smem, *ringX = smem + NSW * WSTAGE;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const bool x_loader = w < 4;
    int nblk = gridDim.x, bid = blockIdx.x;
    if (a.n_xcd > 1 && nblk % a.n_xcd == 0) bid = (bid % a.n_xcd) * (nblk / a.n_xcd) + bid / a.n_xcd;
    const int tb = bid % a.n_tblk, fb = bid / a.n_tblk;
    const int ft0 = fb * FS, tt0 = tb * TS;
    const int z = blockIdx.z;
    const int ktile0 = z * a.ksteps_per_split * 4;
    int ktiles = (a.Kp >> 4) - ktile0;
    if (ktiles > a.ksteps_per_split * 4) ktiles = a.ksteps_per_split * 4;
    const int nsteps = ktiles / BKT;
    const size_t strip_bytes = (size_t)(a.Kp >> 4) * 1024;

    constexpr int MAXL = XLPW > WLPW ? XLPW : WLPW;
    const char *ub[MAXL];
#pragma unroll
    for (int i = 0; i < MAXL; ++i) {
        const int u = (w & 3) + 4 * i, p = u / BKT, kt = u % BKT;
        const char *base;
        if (x_loader) {
            int s_ = tt0 + p;
            if (s_ >= a.n_ttiles) s_ = a.n_ttiles - 1;  // out-of-range strips duplicate a valid one; never stored
            base = (const char *)a.X + (size_t)s_ * strip_bytes;
        } else {
            int s_ = ft0 + (p < FS ? p : FS - 1);
            if (s_ >= a.n_ftiles) s_ = a.n_ftiles - 1;
            base = (const char *)a.W + (size_t)s_ * strip_bytes;
        }
        ub[i] = base + (size_t)(ktile0 + kt) * 1024 + lane * 16;
    }
    auto issue = [&](int ks) {  // this wavefront's share of stage ks of its ring
        if (x_loader) {
            char *dst = ringX + (ks % NSX) * XSTAGE + (w & 3) * 1024;
#pragma unroll
            for (int i = 0; i < XLPW; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ub[i] + (size_t)ks * (BKT * 1024)),
                                                 (__attribute__((address_space(3))) void *)(dst + i * 4096), 16, 0, 0);
        } else {
            char *dst = ringW + (ks % NSW) * WSTAGE + (w & 3) * 1024;
#pragma unroll
            for (int i = 0; i < WLPW; ++i)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ub[i] + (size_t)ks * (BKT * 1024)),
                                                 (__attribute__((address_space(3))) void *)(dst + i * 4096), 16, 0, 0);
        }
    };

    f32x16 acc[FW][TW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    {
        const int pro = x_loader ? NSX - 1 : NSW - 1;
        for (int s_ = 0; s_ < pro; ++s_)
            if (s_ < nsteps) issue(s_);
    }

    f16x8 fa[2][FW], fb_[2][TW];
    const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) char *)ringW + lane * 16;
    const unsigned lds_x = (unsigned)(size_t)(__attribute__((address_space(3))) char *)ringX + (2 * w) * (BKT * 1024) + lane * 16;
    auto read_frags = [&](int buf, int ks, int kt) {
        const unsigned offw = (ks % NSW) * WSTAGE + kt * 1024, offx = (ks % NSX) * XSTAGE + kt * 1024;
#pragma unroll
        for (int i = 0; i < FW; ++i) asm volatile("ds_read_b128 %0, %1" : "=v"(fa[buf][i]) : "v"(lds_w + offw + i * (BKT * 1024)));
#pragma unroll
        for (int j = 0; j < TW; ++j) asm volatile("ds_read_b128 %0, %1" : "=v"(fb_[buf][j]) : "v"(lds_x + offx + j * (BKT * 1024)));
    };
    auto frags_ready = [&](int buf, bool newer_in_flight) {
        if (newer_in_flight) wait_lgkmcnt<FW + TW>();
        else wait_lgkmcnt<0>();
#pragma unroll
        for (int i = 0; i < FW; ++i) asm volatile("" : "+v"(fa[buf][i]));
#pragma unroll
        for (int j = 0; j < TW; ++j) asm volatile("" : "+v"(fb_[buf][j]));
    };
    auto publish_next = [&](int ks) {
        // own loads issued after those of step ks + 1 and allowed to stay in flight
        const int later = nsteps - 2 - ks;
        if (x_loader) {
            if (NSX >= 4 && later >= NSX - 3) wait_vmcnt<(NSX >= 4 ? NSX - 3 : 0) * XLPW>();
            else wait_vmcnt<0>();
        } else {
            const int g_ = later < NSW - 3 ? later : NSW - 3;
            switch (g_) {
                case 5: wait_vmcnt<5 * WLPW>(); break;
                case 4: wait_vmcnt<4 * WLPW>(); break;
                case 3: wait_vmcnt<3 * WLPW>(); break;
                case 2: wait_vmcnt<2 * WLPW>(); break;
                case 1: wait_vmcnt<1 * WLPW>(); break;
                default: wait_vmcnt<0>(); break;
            }
        }
        __builtin_amdgcn_s_barrier();
        const int nxt = ks + (x_loader ? NSX - 1 : NSW - 1);
        if (nxt < nsteps) issue(nxt);
    };
    if (nsteps > 0) {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);
    }
    auto stage = [&](int ks, auto has_next) {
#pragma unroll
        for (int kt = 0; kt < BKT; ++kt) {
            const int c = kt & 1;
            bool newer = true;
            if (kt == BKT - 1) {
                if constexpr (decltype(has_next)::value) {
                    publish_next(ks);
                    read_frags(c ^ 1, ks + 1, 0);
                } else {
                    newer = false;
                }
            } else {
                read_frags(c ^ 1, ks, kt + 1);
            }
            frags_ready(c, newer);
#pragma unroll
            for (int i = 0; i < FW; ++i)
#pragma unroll
                for (int j = 0; j < TW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[c][i], fb_[c][j], acc[i][j], 0, 0, 0);
        }
    };
    for (int ks = 0; ks + 1 < nsteps; ++ks) stage(ks, std::true_type{});
    if (nsteps > 0) stage(nsteps - 1, std::false_type{});
    gemm_epilogue<FW, TW, EPI>(a, acc, ft0, tt0 + 2 * w, z, lane);
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
