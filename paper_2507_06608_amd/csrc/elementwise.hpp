// Small memory-bound kernels around the GEMMs: RMSNorm, rotary embedding + KV append, weight packing, KV page
// layout conversion, the rotary table and the debug unpack.
#pragma once
#include "common.hpp"

namespace nexus {

// ---- RMSNorm: h = x * rsqrt(mean(x^2) + eps) * g, one workgroup per token, fp32 statistics -----------------
// Input row-major [T][d]: bf16 (the layer input), fp32 (the residual stream after attention), or -- fused with the
// end of a split-K output projection -- the S fp32 partial slices of that GEMM plus the bf16 residual, in which
// case the kernel also writes the residual stream x1 = residual + sum of slices (slices added in order, then the
// residual, exactly as splitk_reduce_kernel does).  A fourth input is the end of the previous layer's split-K down
// projection: its S slices plus the fp32 residual x1; the kernel writes the layer output y = bf16(x1 + sum), which
// is this layer's input, and normalises the rounded y -- the same values the reduce kernel followed by the bf16
// norm would produce.  Output half, in P32 tile order (operand of the next GEMM).
enum RmsIn { RMS_IN_BF16 = 0, RMS_IN_F32 = 1, RMS_IN_PARTIAL = 2, RMS_IN_PARTIAL_Y = 3 };
struct RmsPartial {
    const float *partial;  // [S][T][d]
    int S, T;
    const bf16_t *res;     // [T][d]   (RMS_IN_PARTIAL)
    float *x1_out;         // [T][d]   (RMS_IN_PARTIAL)
    const float *res_f32;  // [T][d]   (RMS_IN_PARTIAL_Y)
    bf16_t *y_out;         // [T][d]   (RMS_IN_PARTIAL_Y)
};
// slices summed in order, then the fp32 residual, rounded to bf16 and stored; v receives the rounded values
__device__ __forceinline__ void sum_partial_y8(const RmsPartial &pp, int t, int d, int ci, float (&v)[8]) {
    sum_slices8(pp.partial + (size_t)t * d + 8 * ci, (size_t)pp.T * d, pp.S, v);
    const float4 *rr = (const float4 *)(pp.res_f32 + (size_t)t * d) + 2 * ci;
    const float4 r0 = rr[0], r1 = rr[1];
    const uint4 y = make_uint4(pack2(v[0] + r0.x, v[1] + r0.y), pack2(v[2] + r0.z, v[3] + r0.w), pack2(v[4] + r1.x, v[5] + r1.y),
                               pack2(v[6] + r1.z, v[7] + r1.w));
    ((uint4 *)(pp.y_out + (size_t)t * d))[ci] = y;
    const uint32_t wds[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = bf2f(wds[e] & 0xffff);
        v[2 * e + 1] = bf2f(wds[e] >> 16);
    }
}
template <int MAXC, int IN>  // 8-element chunks per thread, d <= MAXC * 256 * 8
__global__ __launch_bounds__(256) void rmsnorm_kernel(const void *__restrict__ x, const bf16_t *__restrict__ g,
                                                      f16_t *__restrict__ out_p32, int d, int Kp, float eps, RmsPartial pp) {
    __shared__ float red[4];
    const int t = xcd_run_index(blockIdx.x, gridDim.x), tid = threadIdx.x;  // 8 output rows share a cache line
    const int nchunk = d >> 3;
    float v[MAXC][8];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ci = tid + c * 256;
        if (ci < nchunk) {
            if (IN == RMS_IN_F32) {
                const float4 *row = (const float4 *)((const float *)x + (size_t)t * d);
                float4 a0 = row[2 * ci], a1 = row[2 * ci + 1];
                v[c][0] = a0.x, v[c][1] = a0.y, v[c][2] = a0.z, v[c][3] = a0.w;
                v[c][4] = a1.x, v[c][5] = a1.y, v[c][6] = a1.z, v[c][7] = a1.w;
            } else if (IN == RMS_IN_PARTIAL_Y) {
                sum_partial_y8(pp, t, d, ci, v[c]);
            } else if (IN == RMS_IN_PARTIAL) {
                sum_slices8(pp.partial + (size_t)t * d + 8 * ci, (size_t)pp.T * d, pp.S, v[c]);
                uint4 u = ((const uint4 *)(pp.res + (size_t)t * d))[ci];
                uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[c][2 * e] += bf2f(wds[e] & 0xffff);
                    v[c][2 * e + 1] += bf2f(wds[e] >> 16);
                }
                float4 *orow = (float4 *)(pp.x1_out + (size_t)t * d);
                orow[2 * ci] = make_float4(v[c][0], v[c][1], v[c][2], v[c][3]);
                orow[2 * ci + 1] = make_float4(v[c][4], v[c][5], v[c][6], v[c][7]);
            } else {
                const uint4 *row = (const uint4 *)((const bf16_t *)x + (size_t)t * d);
                uint4 u = row[ci];
                uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[c][2 * e] = bf2f(wds[e] & 0xffff);
                    v[c][2 * e + 1] = bf2f(wds[e] >> 16);
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += v[c][e] * v[c][e];
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float inv = rsqrtf(tot / (float)d + eps);
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ci = tid + c * 256;
        if (ci < nchunk) {
            uint4 gu = ((const uint4 *)g)[ci];
            uint32_t gw[4] = {gu.x, gu.y, gu.z, gu.w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = packh2(v[c][2 * e] * inv * bf2f(gw[e] & 0xffff), v[c][2 * e + 1] * inv * bf2f(gw[e] >> 16));
            *(uint4 *)(out_p32 + p32_offset(t, ci * 8, Kp)) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

// The same norm with one wavefront per token, for long batches: the wavefront keeps its whole row in registers
// (MAXC 16-byte chunks per lane, all loaded before the first is used) and the only reduction is a wavefront
// shuffle.  With thousands of rows this moves 1.4x the bytes per second of the workgroup-per-token kernel above
// (8192 rows of 4096: 72 -> 53 us); with a few hundred rows the latter has four times the wavefronts to hide its
// latencies with and wins, above all where the slices of a split-K GEMM are summed in passing (512 rows: 10 us
// against 22).  A workgroup is kRmsWaves = 8 consecutive rows, because 8 rows of the tile-ordered output are one
// 128-byte line (16 bytes of each): the wavefronts lay their normalised rows into LDS (8 rows, up to 128 KiB, one
// barrier) and write whole lines instead of 16-byte pieces of 64 different lines each.
constexpr int kRmsWaves = 8;
template <int MAXC, int IN>  // 8-element chunks per lane, d <= MAXC * 64 * 8
__global__ __launch_bounds__(64 * kRmsWaves) void rmsnorm_wave_kernel(const void *__restrict__ x, const bf16_t *__restrict__ g,
                                                                 f16_t *__restrict__ out_p32, int n_tokens, int d, int Kp, float eps,
                                                                 RmsPartial pp) {
    extern __shared__ uint4 stage[];  // [row][MAXC * 64 + 1 chunks] (+ 1: the transposed reads spread over the banks); sized by the host
    constexpr int SP = MAXC * 64 + 1;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int t0 = xcd_run_index(blockIdx.x, gridDim.x) * kRmsWaves;
    const int t = t0 + w < n_tokens ? t0 + w : n_tokens - 1;  // (a wavefront past the last row touches no row: see nload)
    const bool row_ok = t0 + w < n_tokens;
    const int nchunk = d >> 3;
    const int nload = row_ok ? nchunk : 0;  // a wavefront without a row loads and stores nothing and carries zeros
    float v[MAXC][8];
    if (IN == RMS_IN_BF16) {
        uint4 u[MAXC];
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int ci = lane + c * 64;
            u[c] = make_uint4(0, 0, 0, 0);
            if (ci < nload) u[c] = ((const uint4 *)((const bf16_t *)x + (size_t)t * d))[ci];
        }
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const uint32_t wds[4] = {u[c].x, u[c].y, u[c].z, u[c].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[c][2 * e] = bf2f(wds[e] & 0xffff);
                v[c][2 * e + 1] = bf2f(wds[e] >> 16);
            }
        }
    } else if (IN == RMS_IN_F32) {
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int ci = lane + c * 64;
            float4 a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
            if (ci < nload) {
                const float4 *row = (const float4 *)((const float *)x + (size_t)t * d);
                a0 = row[2 * ci], a1 = row[2 * ci + 1];
            }
            v[c][0] = a0.x, v[c][1] = a0.y, v[c][2] = a0.z, v[c][3] = a0.w;
            v[c][4] = a1.x, v[c][5] = a1.y, v[c][6] = a1.z, v[c][7] = a1.w;
        }
    } else if (IN == RMS_IN_PARTIAL_Y) {
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int ci = lane + c * 64;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[c][e] = 0.f;
            if (ci < nload) sum_partial_y8(pp, t, d, ci, v[c]);
        }
    } else {
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int ci = lane + c * 64;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[c][e] = 0.f;
            if (ci < nload) sum_slices8(pp.partial + (size_t)t * d + 8 * ci, (size_t)pp.T * d, pp.S, v[c]);
        }
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int ci = lane + c * 64;
            if (ci < nload) {
                const uint4 u = ((const uint4 *)(pp.res + (size_t)t * d))[ci];
                const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[c][2 * e] += bf2f(wds[e] & 0xffff);
                    v[c][2 * e + 1] += bf2f(wds[e] >> 16);
                }
                float4 *orow = (float4 *)(pp.x1_out + (size_t)t * d);
                orow[2 * ci] = make_float4(v[c][0], v[c][1], v[c][2], v[c][3]);
                orow[2 * ci + 1] = make_float4(v[c][4], v[c][5], v[c][6], v[c][7]);
            }
        }
    }
    float ss = 0.f;  // chunks past the row hold zeros
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += v[c][e] * v[c][e];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float inv = rsqrtf(ss / (float)d + eps);
    // lane (row r = lane % 8, line lane / 8 of this wavefront's eight) of the write-out: 8 lanes cover one 128-byte line
    const int r_out = lane & 7, li = w * 8 + (lane >> 3);
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ci = lane + c * 64;
        uint4 o4 = make_uint4(0, 0, 0, 0);
        if (ci < nchunk) {
            const uint4 gu = ((const uint4 *)g)[ci];
            const uint32_t gw[4] = {gu.x, gu.y, gu.z, gu.w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = packh2(v[c][2 * e] * inv * bf2f(gw[e] & 0xffff), v[c][2 * e + 1] * inv * bf2f(gw[e] >> 16));
            o4 = make_uint4(o[0], o[1], o[2], o[3]);
        }
        stage[w * SP + ci] = o4;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int co = li + c * 64;
        if (co < nchunk && t0 + r_out < n_tokens) *(uint4 *)(out_p32 + p32_offset(t0 + r_out, co * 8, Kp)) = stage[r_out * SP + co];
    }
}

// ---- rotary table: tab[pos][j] = (cos, sin)(pos * theta^(-2j/hd)), angles in fp64 ------------------------
__global__ void rope_table_kernel(float2 *tab, int n_pos, int half, double theta) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)n_pos * half) return;
    const int pos = (int)(i / half), j = (int)(i % half);
    const double freq = pow(theta, -(double)j / (double)half);
    const double phi = (double)pos * freq;
    tab[i] = make_float2((float)cos(phi), (float)sin(phi));
}

// ---- rotary embedding + KV append ---------------------------------------------------------------------------
// Reads the QKV projection output (half, row-major [T][(Hq+2Hkv)*hd]); rotates q and k at the token's absolute
// position; writes q for the attention kernel and k, v into the token's (page, slot) of the pools.
struct RopeArgs {
    const f16_t *qkv;
    int T, Hq, Hkv, hd;
    const float2 *rope_tab;
    int n_pos;
    // prefill: requests packed, positions prefix_len[r] + local; decode (cu_chunk == null): pos = ctx_len[t]
    const int32_t *cu_chunk;
    const int32_t *pos_base;  // prefix_len or ctx_len
    int n_reqs;
    const int32_t *page_table;
    int max_pages;
    bf16_t *k_pool, *v_pool;
    int n_pages;
    bf16_t *q_out;  // prefill: P32 with request-aligned 32-row tiles; decode: row-major [T][Hq*hd]
    // When the QKV projection was split along K, its S fp32 partial slices [S][T][Hq*hd + 2*Hkv*hd] (+ bias) are
    // summed here instead of by a reduce kernel; the sum is rounded to half first, as that kernel would have.
    const float *partial;
    int S;
    const bf16_t *bias;
};

// The decode side: one workgroup per request's new token (the tokens of a decode batch belong to different requests
// and pages, there is nothing to share between neighbours).
__global__ __launch_bounds__(256) void rope_append_decode_kernel(RopeArgs a) {
    const int t = blockIdx.x;
    const int hd = a.hd, half = hd >> 1, cph = half >> 3;  // chunks of 8 rotary pairs per head
    const int r = t, pos = a.pos_base[t], qrow = t;
    const int qd = a.Hq * hd, kvd = a.Hkv * hd;
    const f16_t *row = a.qkv + (size_t)t * (qd + 2 * kvd);
    int page = -1;
    const int lp = pos >> 4, slot = pos & 15;
    if (lp < a.max_pages) page = a.page_table[(size_t)r * a.max_pages + lp];
    const bool page_ok = (unsigned)page < (unsigned)a.n_pages;
    const int ptab = pos < a.n_pos ? pos : a.n_pos - 1;
    const float2 *tab = a.rope_tab + (size_t)ptab * half;

    const int width = qd + 2 * kvd;
    auto load8 = [&](int col, float (&o)[8]) {
        if (a.partial) {
            sum_slices8(a.partial + (size_t)t * width + col, (size_t)a.T * width, a.S, o);
            if (a.bias) {
                const uint4 b = *(const uint4 *)(a.bias + col);
                const uint32_t bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += bf2f((bw[e >> 1] >> ((e & 1) * 16)) & 0xffff);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = h2f(f2h(o[e]));
        } else {
            const uint4 u = *(const uint4 *)(row + col);
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = h2f((f16_t)((w[e >> 1] >> ((e & 1) * 16)) & 0xffff));
        }
    };
    const int rope_units = (a.Hq + a.Hkv) * cph;
    const int v_units = a.Hkv * (hd >> 3);
    // gridDim.y workgroups share a token's units: a decode batch has too few tokens to put one on every CU
    for (int u = threadIdx.x + 256 * blockIdx.y; u < rope_units + v_units; u += 256 * gridDim.y) {
        if (u < rope_units) {
            const int h = u / cph, c = u % cph;  // head (q heads first, then k heads), pair chunk
            float xl[8], xh[8], ol[8], oh[8];
            load8(h * hd + c * 8, xl);
            load8(h * hd + half + c * 8, xh);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x0 = xl[e], x1 = xh[e];
                const float2 cs = tab[c * 8 + e];
                ol[e] = x0 * cs.x - x1 * cs.y;
                oh[e] = x1 * cs.x + x0 * cs.y;
            }
            uint4 plo = make_uint4(pack2(ol[0], ol[1]), pack2(ol[2], ol[3]), pack2(ol[4], ol[5]), pack2(ol[6], ol[7]));
            uint4 phi = make_uint4(pack2(oh[0], oh[1]), pack2(oh[2], oh[3]), pack2(oh[4], oh[5]), pack2(oh[6], oh[7]));
            if (h < a.Hq) {
                *(uint4 *)(a.q_out + (size_t)qrow * qd + h * hd + c * 8) = plo;
                *(uint4 *)(a.q_out + (size_t)qrow * qd + h * hd + half + c * 8) = phi;
            } else if (page_ok) {
                const int kvh = h - a.Hq;
                bf16_t *blk = a.k_pool + ((size_t)page * a.Hkv + kvh) * (kPage * hd);
                *(uint4 *)(blk + kblk_offset(slot, c * 8)) = plo;
                *(uint4 *)(blk + kblk_offset(slot, half + c * 8)) = phi;
            }
        } else if (page_ok) {
            const int vu = u - rope_units;
            const int kvh = vu / (hd >> 3), c = vu % (hd >> 3);
            float vv[8];
            load8(qd + kvd + kvh * hd + c * 8, vv);
            bf16_t *blk = a.v_pool + ((size_t)page * a.Hkv + kvh) * (kPage * hd);
#pragma unroll
            for (int e = 0; e < 8; ++e) blk[vblk_offset(slot, c * 8 + e, hd)] = f2bf(vv[e]);
        }
    }
}

// The prefill side of the same operation with a workgroup per 8 consecutive chunk tokens of a request (a quarter of
// a 32-row query tile), because 8 is the unit everything it writes comes in: 8 rows of a query tile are one 128-byte
// line (16 bytes of each), 8 tokens one 16-byte V operand, 8 consecutive positions two 64-byte runs of a K block.
// With a workgroup per token every store instruction put 16-byte (V: 2-byte) pieces into 64 different lines; here
// the 8 lanes that share a line are neighbours.  Thread (j = tid % 8, tid / 8): token j of the group, one of 32
// units in flight; a unit is a chunk of 8 rotary pairs of a head (q heads first, then k heads) or 8 value elements.
// The values of a unit pass through LDS to change hands: lane j then holds element j of the unit for the 8 tokens.
// Grid: x = 4 groups per 32-row tile of the request-aligned query rows (at least the batch's tile count), y = the
// workgroups that share a group's units (short batches have too few groups to fill the chip).
__global__ __launch_bounds__(256) void rope_append_prefill_kernel(RopeArgs a) {
    __shared__ uint4 vst[32][9];  // [unit in flight][token] (+ 1: the transposed reads spread over the banks)
    const int b = xcd_run_index(blockIdx.x, gridDim.x);
    const int ti = b >> 2, sub = b & 3;
    int r = 0, tile_base = 0;
    for (;; ++r) {
        if (r >= a.n_reqs) return;
        const int nt = (a.cu_chunk[r + 1] - a.cu_chunk[r] + 31) >> 5;
        if (ti < tile_base + nt) break;
        tile_base += nt;
    }
    const int c0 = a.cu_chunk[r], n_r = a.cu_chunk[r + 1] - c0;
    const int local0 = (ti - tile_base) * 32 + sub * 8;
    if (local0 >= n_r) return;  // the whole workgroup
    const int j = threadIdx.x & 7, ul = threadIdx.x >> 3;
    const bool tok_ok = local0 + j < n_r;
    const int t = c0 + (tok_ok ? local0 + j : n_r - 1);  // (a lane without a token reads the last one's row and stores nothing)
    const int pos0 = a.pos_base[r] + local0, pos = pos0 + j;
    const int qrow = ti * 32 + sub * 8 + j;
    const int hd = a.hd, half = hd >> 1, cph = half >> 3;
    const int qd = a.Hq * hd, kvd = a.Hkv * hd, width = qd + 2 * kvd;
    const f16_t *row = a.qkv + (size_t)t * width;
    auto page_of = [&](int p) {
        const int lp = p >> 4;
        const int page = lp < a.max_pages ? a.page_table[(size_t)r * a.max_pages + lp] : -1;
        return (unsigned)page < (unsigned)a.n_pages ? page : -1;
    };
    const int page = tok_ok ? page_of(pos) : -1;
    const int slot = pos & 15;
    const float2 *tab = a.rope_tab + (size_t)(pos < a.n_pos ? pos : a.n_pos - 1) * half;
    auto load8 = [&](int col, float (&o)[8]) {
        if (a.partial) {
            sum_slices8(a.partial + (size_t)t * width + col, (size_t)a.T * width, a.S, o);
            if (a.bias) {
                const uint4 bb = *(const uint4 *)(a.bias + col);
                const uint32_t bw[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += bf2f((bw[e >> 1] >> ((e & 1) * 16)) & 0xffff);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = h2f(f2h(o[e]));
        } else {
            const uint4 u = *(const uint4 *)(row + col);
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = h2f((f16_t)((w[e >> 1] >> ((e & 1) * 16)) & 0xffff));
        }
    };
    const int rope_units = (a.Hq + a.Hkv) * cph;
    const int uy = 32 * blockIdx.y, ustep = 32 * gridDim.y;  // the units are dealt to gridDim.y workgroups, 32 at a time
    // cph divides 32 (head dimensions 64 and 128): a thread's units all have the same pair chunk, whose eight
    // (cos, sin) it reads once instead of once per head
    const int c = ul % cph;
    float2 cs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = tab[c * 8 + e];
    for (int u = uy + ul; u < rope_units; u += ustep) {
        if (!tok_ok) continue;
        const int h = u / cph;
        float xl[8], xh[8], ol[8], oh[8];
        load8(h * hd + c * 8, xl);
        load8(h * hd + half + c * 8, xh);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x0 = xl[e], x1 = xh[e];
            ol[e] = x0 * cs[e].x - x1 * cs[e].y;
            oh[e] = x1 * cs[e].x + x0 * cs[e].y;
        }
        const uint4 plo = make_uint4(pack2(ol[0], ol[1]), pack2(ol[2], ol[3]), pack2(ol[4], ol[5]), pack2(ol[6], ol[7]));
        const uint4 phi = make_uint4(pack2(oh[0], oh[1]), pack2(oh[2], oh[3]), pack2(oh[4], oh[5]), pack2(oh[6], oh[7]));
        if (h < a.Hq) {
            *(uint4 *)(a.q_out + p32_offset(qrow, h * hd + c * 8, qd)) = plo;
            *(uint4 *)(a.q_out + p32_offset(qrow, h * hd + half + c * 8, qd)) = phi;
        } else if (page >= 0) {
            bf16_t *blk = a.k_pool + ((size_t)page * a.Hkv + (h - a.Hq)) * (kPage * hd);
            *(uint4 *)(blk + kblk_offset(slot, c * 8)) = plo;
            *(uint4 *)(blk + kblk_offset(slot, half + c * 8)) = phi;
        }
    }
    // values: 8 tokens x 8 elements change hands through LDS, then one 16-byte operand per lane when the group is a
    // whole, aligned token group of one page; single elements otherwise (ragged tail, prefix not a multiple of 8)
    const int v_units = a.Hkv * (hd >> 3);
    const bool whole = (pos0 & 7) == 0 && local0 + 8 <= n_r;
    const int page0 = whole ? page_of(pos0) : -1;
    for (int ub = uy; ub < v_units; ub += ustep) {  // uniform trip count: the barriers below are the workgroup's
        const int u = ub + ul;
        const bool unit_ok = u < v_units;
        const int kvh = unit_ok ? u / (hd >> 3) : 0, c = unit_ok ? u % (hd >> 3) : 0;
        float vv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (unit_ok && tok_ok) load8(qd + kvd + kvh * hd + c * 8, vv);
        vst[ul][j] = make_uint4(pack2(vv[0], vv[1]), pack2(vv[2], vv[3]), pack2(vv[4], vv[5]), pack2(vv[6], vv[7]));
        __syncthreads();
        if (unit_ok) {
            bf16_t el[8];  // element j of the unit for tokens 0..7 of the group
#pragma unroll
            for (int k = 0; k < 8; ++k) el[k] = ((const bf16_t *)&vst[ul][k])[j];
            if (whole) {
                if (page0 >= 0) {
                    bf16_t *blk = a.v_pool + ((size_t)page0 * a.Hkv + kvh) * (kPage * hd);
                    const uint4 o = make_uint4((uint32_t)el[0] | ((uint32_t)el[1] << 16), (uint32_t)el[2] | ((uint32_t)el[3] << 16),
                                               (uint32_t)el[4] | ((uint32_t)el[5] << 16), (uint32_t)el[6] | ((uint32_t)el[7] << 16));
                    *(uint4 *)(blk + vblk_offset(pos0 & 15, c * 8 + j, hd)) = o;
                }
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    if (local0 + k >= n_r) break;
                    const int pk = page_of(pos0 + k);
                    if (pk >= 0) (a.v_pool + ((size_t)pk * a.Hkv + kvh) * (kPage * hd))[vblk_offset((pos0 + k) & 15, c * 8 + j, hd)] = el[k];
                }
            }
        }
        __syncthreads();
    }
}

// ---- weight packing: bf16 row-major [N][K] -> half P32 [round_up(N,32)][Kp], zero padded -----------------------
// bf16 -> half is exact for |w| >= 2^-14 and off by at most 2^-25 below that.
// interleave_F > 0 reorders gate/up rows so that packed strip s holds gate rows [16s, 16s+16) followed by up rows
// [16s, 16s+16): in the 32x32 MFMA tile of the strip a lane then holds a gate value and, two register quads
// later, its up value.
__global__ void pack_weight_kernel(const bf16_t *__restrict__ src, f16_t *__restrict__ dst, int N, int K, int Kp,
                                   int interleave_F) {
    const int Np = round_up(N, 32);
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int kchunks = Kp >> 3;
    if (idx >= (size_t)Np * kchunks) return;
    const int n = (int)(idx / kchunks), k = (int)(idx % kchunks) * 8;
    int srow = n;
    if (interleave_F > 0) {
        const int strip = n >> 5, r = n & 31;
        srow = (r >> 4) * interleave_F + strip * 16 + (r & 15);
    }
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N && k < K) {
        if (k + 8 <= K && (K & 7) == 0) {
            v = *(const uint4 *)(src + (size_t)srow * K + k);
        } else {
            bf16_t tmp[8];
            for (int e = 0; e < 8; ++e) tmp[e] = (k + e < K) ? src[(size_t)srow * K + k + e] : (bf16_t)0;
            v = *(uint4 *)tmp;
        }
    }
    uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) wds[e] = packh2(bf2f(wds[e] & 0xffff), bf2f(wds[e] >> 16));
    *(uint4 *)(dst + p32_offset(n, k, Kp)) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
}

// ---- KV page layout conversion (canonical [pages][Hkv][16][hd] <-> private blocks) -------------------------
template <bool IMPORT>
__global__ void kv_convert_kernel(bf16_t *k_priv, bf16_t *v_priv, bf16_t *k_canon, bf16_t *v_canon, int n_blocks /*pages*Hkv*/,
                                  int hd) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int per_blk = kPage * hd;
    if (idx >= (size_t)n_blocks * per_blk) return;
    const size_t blk = idx / per_blk;
    const int e = (int)(idx % per_blk), tok = e / hd, i = e % hd;
    const size_t ko = blk * per_blk + kblk_offset(tok, i), vo = blk * per_blk + vblk_offset(tok, i, hd);
    if (IMPORT) {
        k_priv[ko] = k_canon[idx];
        v_priv[vo] = v_canon[idx];
    } else {
        k_canon[idx] = k_priv[ko];
        v_canon[idx] = v_priv[vo];
    }
}

// ---- debug: 16-bit P32 or row-major buffer -> fp32 row-major ----------------------------------------------------
// kind: 0 = half P32, 1 = bf16 P32, 2 = half row-major, 3 = bf16 row-major
__global__ void debug_to_f32_kernel(const unsigned short *__restrict__ src, float *__restrict__ dst, int rows, int K, int Kp, int kind) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)rows * K) return;
    const int r = (int)(idx / K), k = (int)(idx % K);
    const unsigned short v = kind < 2 ? src[p32_offset(r, k, Kp)] : src[idx];
    dst[idx] = (kind & 1) ? bf2f(v) : h2f(v);
}

// ---- CU probe: where does each workgroup of a masked stream run? -------------------------------------------
__global__ void cu_probe_kernel(int32_t *counts) {
    uint32_t hw_id, xcc_id;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw_id));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc_id));
    if (threadIdx.x == 0) {
        const int cu = (hw_id >> 8) & 0xf, se = (hw_id >> 13) & 0x7;  // CU_ID and SE_ID fields of HW_ID
        atomicAdd(&counts[(xcc_id & 7) * 128 + se * 16 + cu], 1);
    }
    // a little work so that workgroups spread over the CUs instead of draining through the first one
    float acc = (float)threadIdx.x;
    for (int i = 0; i < 2000; ++i) acc = acc * 1.0001f + 0.5f;
    if (acc == 12345.678f) counts[0] = -1;
}

}  // namespace nexus
