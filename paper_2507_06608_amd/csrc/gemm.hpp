// bf16 MFMA projection GEMMs of the layer (Eq. 1-3): Y[T][N] = X[T][K] * W[N][K]^T with fused epilogues.
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
#include "common.hpp"

namespace nexus {

enum GemmEpi : int {
    EPI_ROWMAJOR = 0,  // out[t][f] = bf16(acc (+ bias[f]))
    EPI_RESIDUAL = 1,  // out[t][f] = bf16(res[t][f] + acc)
    EPI_SWIGLU = 2,    // weight strips alternate gate/up; out_p32[t][f] = bf16(silu(gate) * up)
    EPI_PARTIAL = 3    // partial[z][t][n] = acc (fp32), finished by splitk_reduce
};

struct GemmArgs {
    const bf16_t *W;   // P32 [n_ftiles*32][Kp]
    const bf16_t *X;   // P32 [n_ttiles*32][Kp]
    int n_ftiles, n_ttiles, Kp;
    int ksteps_per_split;  // K steps of 64 handled by one z-slice
    int T, N;              // valid tokens; N = n_ftiles * 32 (packed row count)
    bf16_t *out;           // row-major [T][ld_out]
    const bf16_t *res;     // row-major [T][ld_out]
    const bf16_t *bias;    // [N] or null
    int ld_out;
    bf16_t *out_p32;       // EPI_SWIGLU destination, P32 with out_Kp
    int out_Kp;
    float *partial;        // [S][T][N]
    int n_tblk;            // token blocks in the grid
    int n_xcd;             // XCDs the launch is spread over (tile-order remap), >= 1
};

constexpr int kGemmBK = 64;         // k per main-loop step (4 P32 tiles)
constexpr int kStripStage = 4096;   // bytes of one 32-row strip per step

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

template <int FS, int TS, int WF, int WT, int EPI>
__global__ __launch_bounds__(256) void gemm_p32_kernel(GemmArgs a) {
    static_assert(WF * WT == 4, "four waves per block");
    static_assert(FS % WF == 0 && TS % WT == 0, "whole tiles per wave");
    static_assert((FS / WF) % 2 == 0, "a wave needs gate/up strip pairs (and the SwiGLU epilogue reads acc[i + 1])");
    constexpr int FW = FS / WF, TW = TS / WT;
    constexpr int NP = FS + TS;
    constexpr int STAGE = NP * kStripStage;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wf = w % WF, wt = w / WF;

    // Tile order: blocks that share weight strips should meet in one XCD's L2.  Workgroups are dealt to XCDs
    // round-robin, so block b lands on XCD b % n_xcd; give each XCD a contiguous range of logical tiles.
    int nblk = gridDim.x, bid = blockIdx.x;
    if (a.n_xcd > 1 && nblk % a.n_xcd == 0) bid = (bid % a.n_xcd) * (nblk / a.n_xcd) + bid / a.n_xcd;
    const int tb = bid % a.n_tblk, fb = bid / a.n_tblk;
    const int ft0 = fb * FS, tt0 = tb * TS;
    const int z = blockIdx.z;
    const int kstep0 = z * a.ksteps_per_split;
    int nsteps = a.Kp / kGemmBK - kstep0;
    if (nsteps > a.ksteps_per_split) nsteps = a.ksteps_per_split;

    const size_t strip_bytes = (size_t)(a.Kp >> 4) * 1024;
    const char *src[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        if (p < FS) {
            int s = ft0 + p;
            if (s >= a.n_ftiles) s = a.n_ftiles - 1;  // out-of-range strips duplicate a valid one; never stored
            src[p] = (const char *)a.W + (size_t)s * strip_bytes;
        } else {
            int s = tt0 + (p - FS);
            if (s >= a.n_ttiles) s = a.n_ttiles - 1;
            src[p] = (const char *)a.X + (size_t)s * strip_bytes;
        }
        src[p] += (size_t)kstep0 * kStripStage + tid * 16;
    }

    f32x16 acc[FW][TW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 stage_regs[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) stage_regs[p] = *(const u32x4 *)(src[p]);
#pragma unroll
    for (int p = 0; p < NP; ++p) *(u32x4 *)(smem + p * kStripStage + tid * 16) = stage_regs[p];
    __syncthreads();

    for (int ks = 0; ks < nsteps; ++ks) {
        const int cur = ks & 1;
        const bool more = ks + 1 < nsteps;
        if (more) {
#pragma unroll
            for (int p = 0; p < NP; ++p) stage_regs[p] = *(const u32x4 *)(src[p] + (size_t)(ks + 1) * kStripStage);
        }
        const char *sW = smem + cur * STAGE + (wf * FW) * kStripStage + lane * 16;
        const char *sX = smem + cur * STAGE + (FS + wt * TW) * kStripStage + lane * 16;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            bf16x8 fa[FW], fb_[TW];
#pragma unroll
            for (int i = 0; i < FW; ++i) fa[i] = *(const bf16x8 *)(sW + i * kStripStage + kt * 1024);
#pragma unroll
            for (int j = 0; j < TW; ++j) fb_[j] = *(const bf16x8 *)(sX + j * kStripStage + kt * 1024);
#pragma unroll
            for (int i = 0; i < FW; ++i)
#pragma unroll
                for (int j = 0; j < TW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb_[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
#pragma unroll
            for (int p = 0; p < NP; ++p) *(u32x4 *)(smem + (cur ^ 1) * STAGE + p * kStripStage + tid * 16) = stage_regs[p];
        }
        __syncthreads();
    }

    // ---- epilogue: lane owns token column (lane % 32); register 4*b + j is feature row 8*b + 4*(lane/32) + j ----
    const int g = lane >> 5;
#pragma unroll
    for (int j = 0; j < TW; ++j) {
        const int t = (tt0 + wt * TW + j) * 32 + (lane & 31);
        if (t >= a.T) continue;
        if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int i = 0; i < FW; i += 2) {
                const int ft = ft0 + wf * FW + i;
                if (ft >= a.n_ftiles) continue;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int f = (ft >> 1) * 32 + 8 * b + 4 * g;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = silu_f(acc[i][j][4 * b + e]) * acc[i + 1][j][4 * b + e];
                    uint2 o = {pack2(v[0], v[1]), pack2(v[2], v[3])};
                    *(uint2 *)(a.out_p32 + p32_offset(t, f, a.out_Kp)) = o;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < FW; ++i) {
                const int ft = ft0 + wf * FW + i;
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
                    } else {
                        if constexpr (EPI == EPI_ROWMAJOR) {
                            if (a.bias) {
                                uint2 bb = *(const uint2 *)(a.bias + f);
                                v[0] += bf2f(bb.x & 0xffff), v[1] += bf2f(bb.x >> 16);
                                v[2] += bf2f(bb.y & 0xffff), v[3] += bf2f(bb.y >> 16);
                            }
                        } else {
                            uint2 rr = *(const uint2 *)(a.res + (size_t)t * a.ld_out + f);
                            v[0] += bf2f(rr.x & 0xffff), v[1] += bf2f(rr.x >> 16);
                            v[2] += bf2f(rr.y & 0xffff), v[3] += bf2f(rr.y >> 16);
                        }
                        uint2 o = {pack2(v[0], v[1]), pack2(v[2], v[3])};
                        *(uint2 *)(a.out + (size_t)t * a.ld_out + f) = o;
                    }
                }
            }
        }
    }
}

// Finishes a split-K GEMM: sums the S fp32 partials in slice order and applies the epilogue.
// One thread per (token, 4 consecutive packed rows).
struct ReduceArgs {
    const float *partial;  // [S][T][N]
    int S, T, N;
    bf16_t *out;
    const bf16_t *res;
    const bf16_t *bias;
    int ld_out;
    bf16_t *out_p32;
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
        uint2 o = {pack2(silu_f(gsum[0]) * usum[0], silu_f(gsum[1]) * usum[1]),
                   pack2(silu_f(gsum[2]) * usum[2], silu_f(gsum[3]) * usum[3])};
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
        } else {
            uint2 rr = *(const uint2 *)(a.res + (size_t)t * a.ld_out + n);
            v[0] += bf2f(rr.x & 0xffff), v[1] += bf2f(rr.x >> 16), v[2] += bf2f(rr.y & 0xffff), v[3] += bf2f(rr.y >> 16);
        }
        uint2 o = {pack2(v[0], v[1]), pack2(v[2], v[3])};
        *(uint2 *)(a.out + (size_t)t * a.ld_out + n) = o;
    }
}

}  // namespace nexus
