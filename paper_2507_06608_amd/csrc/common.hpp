// Shared device-side definitions of the gfx950 kernels: vector types, the MFMA operand tile order used for every
// GEMM operand ("P32"), and the private KV page layouts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nexus {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // 16-byte staging register
typedef unsigned short bf16_t;  // raw storage of a bfloat16
typedef unsigned short f16_t;   // raw storage of an IEEE half

constexpr int kWave = 64;
constexpr int kPage = 16;  // tokens per KV page

// ---- bf16 <-> fp32 (round to nearest even; NaN kept quiet) ------------------------------------------------
__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16); }

// ---- fp16 <-> fp32 (round to nearest even) ------------------------------------------------------------------
// GEMM operands (normalised activations, attention output, SwiGLU activation, packed weights) are IEEE half, not
// bfloat16: the matrix unit runs both at the same rate, and the three extra mantissa bits cut the operand
// rounding error by 8x, which the elementwise parity bar needs once the hidden size reaches the thousands.
// The KV cache, the rotated queries and the layer's input and output stay bfloat16.
__device__ __forceinline__ float h2f(f16_t v) {
    _Float16 h;
    __builtin_memcpy(&h, &v, 2);
    return (float)h;
}
__device__ __forceinline__ f16_t f2h(float f) {
    _Float16 h = (_Float16)f;
    f16_t v;
    __builtin_memcpy(&v, &h, 2);
    return v;
}
__device__ __forceinline__ uint32_t packh2(float lo, float hi) { return (uint32_t)f2h(lo) | ((uint32_t)f2h(hi) << 16); }

// ---- P32: MFMA-operand tile order of a [rows][K] matrix ----------------------------------------------------
// The matrix is cut into tiles of 32 rows x 16 k (1 KiB).  Inside a tile the 64 lanes of a wavefront each own
// 8 consecutive k of one row: lane = row % 32 + 32 * ((k % 16) / 8).  That is exactly the register image of one
// operand of v_mfma_f32_32x32x16_bf16, so a wave loads a tile with one 16-byte access per lane at lane * 16, fully
// coalesced from global memory and conflict-free from LDS.  Tiles of one 32-row strip are contiguous along k;
// Kp (the padded K) is a multiple of 64 and padding holds zeros.
__host__ __device__ __forceinline__ int round_up(int v, int m) { return (v + m - 1) / m * m; }
__host__ __device__ __forceinline__ int p32_kp(int K) { return round_up(K, 64); }
__host__ __device__ __forceinline__ size_t p32_offset(int r, int k, int Kp) {
    return ((size_t)(r >> 5) * (size_t)(Kp >> 4) + (size_t)(k >> 4)) * 512 + (size_t)((r & 31) + 32 * ((k >> 3) & 1)) * 8 +
           (size_t)(k & 7);
}
__host__ __device__ __forceinline__ size_t p32_elems(int rows, int K) { return (size_t)round_up(rows, 32) * p32_kp(K); }

// ---- private KV page layouts (one (page, kv head) block = 16 tokens x hd) ---------------------------------
// Both attention kernels compute S^T = K Q^T and then feed the S^T accumulators, as they stand, into O^T = V^T P^T.
// The accumulator layout of the MFMA gives a lane 4 consecutive rows of each S^T tile; two tiles give it 8
// probabilities, which must be 8 consecutive tokens so that the matching V^T operand is one 16-byte read.
//   K block: [hd / 8][16 slots][8], token t in slot kslot(t) = t with bits 2 and 3 swapped: slots 0..7 hold
//            tokens {0..3, 8..11}, slots 8..15 tokens {4..7, 12..15}; an MFMA operand row is a slot, 16 B per lane,
//            and 8 consecutive slots (one tile's share of a page) are 128 contiguous bytes.
//   V block: [2 token groups][hd][8 tokens]: a lane reads hd row r of token group g as one 16-byte operand.
__host__ __device__ __forceinline__ int kslot(int tok) { return (tok & 3) | ((tok & 8) >> 1) | ((tok & 4) << 1); }
__host__ __device__ __forceinline__ int kblk_offset(int tok, int i) { return ((i >> 3) * kPage + kslot(tok)) * 8 + (i & 7); }
__host__ __device__ __forceinline__ int vblk_offset(int tok, int i, int hd) { return ((tok >> 3) * hd + i) * 8 + (tok & 7); }

// max over the lane pair (l, l ^ 32) in both lanes: the half-wave swap instruction of gfx950 puts the low halves
// of its two operands into one result and the high halves into the other, without the LDS round trip of a
// generic shuffle.
__device__ __forceinline__ float xor32_max(float x) {
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Workgroups are dealt to the 8 XCDs round-robin.  Where neighbouring work items write pieces of the same cache
// lines (token rows of a tile-ordered matrix: 8 rows are one 128-byte line), item = block index assembles every line
// from partial writes out of 8 different L2s.  This permutation of [0, n) gives each XCD runs of 32 (or, for short
// grids, 8) consecutive items instead: inside every aligned group of 256 (64) blocks, the blocks of one XCD take
// consecutive items.  The tail that fills no whole group keeps its order.
__host__ __device__ __forceinline__ int xcd_run_index(int b, int n) {
    if ((b | 255) < n) return (b & ~255) | ((b & 7) << 5) | ((b >> 3) & 31);
    if ((b | 63) < n) return (b & ~63) | ((b & 7) << 3) | ((b >> 3) & 7);
    return b;
}

// Sum of the S fp32 slices of a split-K GEMM at one 8-element (or 4-element) position, slices added in order.  The
// loads of all slices are issued before the first addition (the loop is unrolled over the largest split count with
// the absent slices predicated off): one memory latency for the sum, not one per slice.
constexpr int kMaxSlices = 8;
__device__ __forceinline__ void sum_slices8(const float *first, size_t slice_stride, int S, float (&o)[8]) {
    float4 a[kMaxSlices][2];
#pragma unroll
    for (int s = 0; s < kMaxSlices; ++s)
        if (s < S) {
            const float4 *p = (const float4 *)(first + (size_t)s * slice_stride);
            a[s][0] = p[0], a[s][1] = p[1];
        }
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxSlices; ++s)
        if (s < S) {
            o[0] += a[s][0].x, o[1] += a[s][0].y, o[2] += a[s][0].z, o[3] += a[s][0].w;
            o[4] += a[s][1].x, o[5] += a[s][1].y, o[6] += a[s][1].z, o[7] += a[s][1].w;
        }
}
__device__ __forceinline__ void sum_slices4(const float *first, size_t slice_stride, int S, float (&o)[4]) {
    float4 a[kMaxSlices];
#pragma unroll
    for (int s = 0; s < kMaxSlices; ++s)
        if (s < S) a[s] = *(const float4 *)(first + (size_t)s * slice_stride);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxSlices; ++s)
        if (s < S) o[0] += a[s].x, o[1] += a[s].y, o[2] += a[s].z, o[3] += a[s].w;
}

}  // namespace nexus
