// Runtime of the partitioned prefill/decode step: context, workspace, packed weights, CU-masked stream pairs,
// the two phase chains, the mixed step, the split profiler and the C ABI declared in include/nexus.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <new>
#include <vector>

#include "../../include/nexus.h"
#include "attn_decode.hpp"
#include "attn_prefill.hpp"
#include "common.hpp"
#include "elementwise.hpp"
#include "gemm.hpp"
#include "status.hpp"

using namespace nexus;

// ---------------------------------------------------------------------------------------------- errors
#define HIP_TRY(expr)                                                                                              \
    do {                                                                                                           \
        hipError_t e_ = (expr);                                                                                    \
        if (e_ != hipSuccess) return fail(NEXUS_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)
#define NX_TRY(expr)             \
    do {                         \
        int s_ = (expr);         \
        if (s_ != NEXUS_OK) return s_; \
    } while (0)

// ---------------------------------------------------------------------------------------------- static scratch
// Workspace of nexus_decode_step_noalloc: device memory that exists from the moment the library is loaded, so the
// call allocates nothing.  One copy per GPU, shared by every context on that GPU, held until the process ends.  In
// host code the array's name is only a handle: its device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static unsigned char *g_scratch_ptr[kMaxDevices] = {};

// `device` must be current.
static int scratch_address(int device, unsigned char **out) {
    if (device < 0 || device >= kMaxDevices) return fail(NEXUS_EINVAL, "device %d outside [0, %d)", device, kMaxDevices);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(NEXUS_EHIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", device, hipGetErrorString(e));
        g_scratch_ptr[device] = (unsigned char *)p;
    }
    *out = g_scratch_ptr[device];
    return NEXUS_OK;
}

// Clears a byte range (a multiple of 16 bytes, 16-byte aligned) with a kernel: usable where a memset node is not.
__global__ __launch_bounds__(256) void scratch_clear_kernel(uint4 *p, size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) p[i] = uint4{0u, 0u, 0u, 0u};
}

// ---------------------------------------------------------------------------------------------- context
struct LayerW {
    bf16_t *g1 = nullptr, *g2 = nullptr, *bqkv = nullptr;
    f16_t *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wdown = nullptr;  // half, P32
    bool loaded = false;
};

struct PhaseWs {
    int maxT = 0;
    f16_t *h = nullptr;      // half P32 [maxT][hidden]   RMSNorm output (both norms)
    f16_t *qkv = nullptr;    // half row-major [maxT][n_qkv]
    bf16_t *q = nullptr;     // bf16, rotated; prefill: P32, request-aligned tiles; decode: row-major
    f16_t *attn = nullptr;   // half P32 [maxT][q_dim]
    float *x1 = nullptr;     // fp32 row-major [maxT][hidden]: residual stream after attention
    f16_t *act = nullptr;    // half P32 [maxT][ffn]
    bf16_t *xbuf[2] = {nullptr, nullptr};  // layer ping-pong, row-major [maxT][hidden]
    float *partial = nullptr;
    size_t partial_elems = 0;
    float *part_o = nullptr, *part_ml = nullptr;  // decode attention split results
    int max_spans = 0;
    int q_rows = 0;
};

struct Layout {
    int p_cus = 0, d_cus = 0;  // 0/0 = unpartitioned
    hipStream_t sp = nullptr, sd = nullptr;
    int p_xcd = 8, d_xcd = 8;  // XCDs each stream is spread over (tile-order hint)
    long last_use = 0;
};
// Partitioned stream pairs are kept alive once created (up to max_layouts of them, least recently used retired
// beyond) and switched by pointer.  Every stream is a queue; a process has fewer hardware queues than a full set of
// pairs has streams and the rest are time-multiplexed: measured on MI355X, back-to-back steps run 2-3.5 % slower
// with seven pairs alive than with one (steps timed one at a time do not differ), which is what
// nexus_retire_cu_splits is for.

struct TraceRec {
    hipEvent_t a, b;
};

struct nexus_ctx {
    nexus_model_desc m{};
    nexus_limits lim{};
    int device = 0, n_cus = 0, n_xcd = 8, cus_per_xcd = 32;
    bool allow_p256 = true;
    int force_tile = 0;  // test hook: 256 = 256 x 256 tiles wherever the shape allows, 384 = 256 x 128, 320 = 320 x 256, 128
    int q_dim = 0, kv_dim = 0, n_qkv = 0;
    std::vector<LayerW> layers;
    PhaseWs ws[2];
    float2 *rope_tab = nullptr;
    hipStream_t s_main = nullptr;
    std::map<long, Layout> layouts;
    Layout *cur = nullptr;
    long use_clock = 0;
    bool bits_xcd_major = false;  // CU-mask bit order (see make_mask)
    hipEvent_t ev_fork = nullptr, ev_caller = nullptr, ev_sp0 = nullptr, ev_sp1 = nullptr, ev_sd0 = nullptr, ev_hand = nullptr;
    // automatic handover: phase times of recent steps, read back once those steps have completed (two sets of events,
    // so that a step can be enqueued while the one before it still runs)
    struct HandoverSample {
        hipEvent_t p0 = nullptr, d0 = nullptr, ph = nullptr, d1 = nullptr;  // prefill start, decode start, end of the prefill head, decode end
        Layout *layout = nullptr;
        int head_layers = 0;
        bool pending = false;
    } ho_sample[2];
    int ho_next = 0;
    Layout *ho_layout = nullptr;              // layout the estimates below were measured on
    float ho_decode_ms = 0.f, ho_head_layer_ms = 0.f;
    int last_handover_layer = 0;
    // ev_ph1[phase]: completion of the last launch that used the phase's workspace (single-phase call, mixed step or
    // fused step), recorded on whatever stream it ran on; every later launch on another stream waits for it, so steps
    // stay ordered across a change of layout.  ev_ph0[phase]: start of the last single-phase call.
    hipEvent_t ev_ph0[2] = {nullptr, nullptr}, ev_ph1[2] = {nullptr, nullptr};
    bool ph_recorded[2] = {false, false};
    bool ph_timed[2] = {false, false};               // ev_ph0 belongs to the same launch as ev_ph1
    hipStream_t done_stream[2] = {nullptr, nullptr};  // stream ev_ph1[phase] was recorded on
    int max_layouts = 8;                              // partitioned stream pairs kept alive (7 = every split in steps of 32 CUs)
    bool debug_checks = false;                        // validate device-side lengths and page ids on the host before launching
    // tracing
    int trace_phase = -1, trace_kernel = -1;
    std::vector<TraceRec> trace_pool;
    size_t trace_used = 0;
    int32_t *probe_counts = nullptr;
    unsigned char *scratch_dev = nullptr;  // this GPU's copy of the static scratch array
};

struct DeviceGuard {
    int prev = -1;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        if (prev != dev) (void)hipSetDevice(dev);
        else prev = -1;
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

template <typename T>
static int dev_alloc(T **p, size_t elems, bool zero) {
    *p = nullptr;
    if (elems == 0) elems = 1;
    hipError_t e = hipMalloc((void **)p, elems * sizeof(T));
    if (e != hipSuccess) return fail(NEXUS_ENOMEM, "hipMalloc of %zu bytes failed: %s", elems * sizeof(T), hipGetErrorString(e));
    if (zero) HIP_TRY(hipMemset(*p, 0, elems * sizeof(T)));
    return NEXUS_OK;
}

// ---------------------------------------------------------------------------------------------- GEMM planning
// Tile shapes (features x tokens), wavefronts, k per stage, ring depth.  Measured on MI355X: 128x128 tiles with
// several workgroups per CU beat 256x256 at the token counts of a prefill chunk (and quantise far better on a CU
// share); a batch of at most 128 tokens (a decode batch, a short chunk) streams the weights once and wants many
// small workgroups whose rings together keep about 100 KiB per CU in flight: one CU draws at most about 50 GB/s
// from HBM, so a decode share of the chip is bound by per-CU bytes in flight, not by the HBM interface.
enum GemmVariant {
    GV_P128 = 0,  // gemm_dl_kernel, 128 x 128, 4 waves, 32-wide stages, 64 KiB ring: two workgroups per CU
    GV_P256,      // gemm_dl_kernel, 256 x 256, 8 waves, 128 KiB ring: half the LDS and L2 traffic per flop, for GEMMs
                  //   with several such tiles per CU of the share (same per-element summation order as GV_P128)
    GV_P256x128,  // gemm_dl_kernel, 256 features x 128 tokens, 4 waves of 4 x 2 MFMA tiles, 96 KiB ring, one workgroup per
                  //   CU: between the two in traffic per flop, for grids that the 256 x 256 tiles quantise badly
    GV_S64,       // gemm_stream_kernel, 128 features x 64 tokens, 4 waves: decode batches of 33..64
    GV_S32,       // gemm_stream_kernel, 128 features x 32 tokens, 4 waves: decode batches of at most 32
    GV_S64W,      // gemm_stream_kernel, 256 features x 64 tokens (two feature strips per wave): on a small CU share
                  //   every workgroup re-reads the activations through the same per-CU load path as the weights, and
                  //   twice the features per activation byte is worth more than twice the workgroups
    GV_S128,      // gemm_stream_kernel, 128 features x 128 tokens, 4 waves: batches of 65..128 tokens (a full decode
                  //   pool, a short prefill chunk), still closer to a sweep over the weights than to a tiled GEMM
    GV_S128W,     // gemm_stream_kernel, 256 features x 128 tokens, 8 waves sharing the activation tiles
    GV_R64,       // gemm_dl_kernel with the extent of GV_S64 / GV_S32: k ranges shorter than the streaming
    GV_R32,       //   kernel's pipeline (hidden sizes below 128)
    GV_P320,      // gemm_dl_kernel, 320 features x 256 tokens, 8 waves of 5 x 2 MFMA tiles, 144 KiB ring: for a QKV
                  //   projection whose width is a multiple of 320 (10240 of the 70B-shaped layer: 256 tiles for a
                  //   2048-token chunk, one round of the whole chip where 256 x 256 tiles need a round and a quarter)
    GV_COUNT
};
struct GemmPlan {
    int variant, S, ksteps_per_split, FS, TS;
};
constexpr int kChipCUs = 256;  // the plan is sized for the whole chip, whatever share the phase runs on

// Depends on the problem only (never on the CU share): S fixes the summation order, so results are bit-identical
// across layouts.  Decode GEMMs are cut along K until there are about 200 workgroups (800 wavefronts, each
// with its own weight stream in flight); measured on MI355X, more slices cost more in partial-sum traffic than
// they gain.
static GemmPlan plan_gemm(int T, int n_ftiles, int Kp) {
    const int ksteps = Kp / kGemmBK;
    const int nt = (T + 31) / 32;
    GemmPlan p{};
    int min_ksteps;
    if (T <= 32) {
        p.variant = GV_S32, p.FS = 4, p.TS = 1, min_ksteps = 8;
    } else if (T <= 64) {
        p.variant = GV_S64, p.FS = 4, p.TS = 2, min_ksteps = 8;
    } else if (T <= 128) {
        p.variant = GV_S128, p.FS = 4, p.TS = 4, min_ksteps = 8;
    } else {
        p.variant = GV_P128, p.FS = 4, p.TS = 4, min_ksteps = 16;
    }
    const int blocks = ((n_ftiles + p.FS - 1) / p.FS) * ((nt + p.TS - 1) / p.TS);
    int S = 1;
    if (p.variant != GV_P128) {
        while (S < 8 && blocks * S < (3 * kChipCUs) / 4) S *= 2;
    } else if (blocks < (3 * kChipCUs) / 4) {
        S = std::min(4, (kChipCUs + blocks / 2) / blocks);
    }
    while (S > 1 && ksteps / S < min_ksteps) --S;
    p.ksteps_per_split = (ksteps + S - 1) / S;
    p.S = (ksteps + p.ksteps_per_split - 1) / p.ksteps_per_split;
    return p;
}

template <int FS, int TS, int WF, int WT, int BKT, int NST, int EPI, bool ASM_READS = true, int NWL = 0, bool BUF_LOADS = false>
static hipError_t launch_gemm_t(const GemmArgs &a, dim3 grid, hipStream_t s) {
    constexpr int smem = NST * (FS + TS) * BKT * 1024;
    static bool attr_done = false;  // one context thread at a time (see header)
    auto kern = gemm_dl_kernel<FS, TS, WF, WT, BKT, NST, EPI, ASM_READS, NWL, BUF_LOADS>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64 * WF * WT), smem, s, a);
    return hipGetLastError();
}

constexpr int kStreamDepth = 2;  // stages of weight tiles a streaming wavefront keeps in flight

template <int FW, int TW, int NW, int BKT, int DST, int EPI>
static hipError_t launch_gemm_stream_t(const GemmArgs &a, dim3 grid, hipStream_t s) {
    constexpr int smem = (DST + 1) * TW * BKT * 1024;
    static bool attr_done = false;
    auto kern = gemm_stream_kernel<FW, TW, NW, BKT, DST, EPI>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64 * NW), smem, s, a);
    return hipGetLastError();
}

template <int EPI>
static hipError_t launch_gemm_v(int variant, const GemmArgs &a, dim3 grid, hipStream_t s) {
    switch (variant) {
        case GV_P128: return launch_gemm_t<4, 4, 2, 2, 2, 4, EPI>(a, grid, s);
        case GV_P256:  // buffer loads address an operand matrix with 32-bit offsets
            if ((size_t)a.n_ftiles * a.Kp * 64 < ((size_t)1 << 32) && (size_t)a.n_ttiles * a.Kp * 64 < ((size_t)1 << 32))
                return launch_gemm_t<8, 8, 4, 2, 2, 4, EPI, true, 4, true>(a, grid, s);
            return launch_gemm_t<8, 8, 4, 2, 2, 4, EPI, true, 4, false>(a, grid, s);
        case GV_P256x128: return launch_gemm_t<8, 4, 2, 2, 2, 4, EPI>(a, grid, s);
        case GV_P320:  // planned for the row-major epilogue and operands below 4 GiB only
            if constexpr (EPI == EPI_ROWMAJOR) return launch_gemm_t<10, 8, 2, 4, 2, 4, EPI, true, 4, true>(a, grid, s);
            return hipErrorInvalidValue;
        case GV_S64: return launch_gemm_stream_t<1, 2, 4, 4, kStreamDepth, EPI>(a, grid, s);
        case GV_S32: return launch_gemm_stream_t<1, 1, 4, 4, kStreamDepth, EPI>(a, grid, s);
        case GV_S64W: return launch_gemm_stream_t<2, 2, 4, 4, kStreamDepth, EPI>(a, grid, s);
        case GV_S128: return launch_gemm_stream_t<1, 4, 4, 4, kStreamDepth, EPI>(a, grid, s);
        case GV_S128W: return launch_gemm_stream_t<1, 4, 8, 4, kStreamDepth, EPI>(a, grid, s);
        case GV_R64: return launch_gemm_t<4, 2, 2, 2, 4, 4, EPI, false>(a, grid, s);
        default: return launch_gemm_t<4, 1, 4, 1, 4, 4, EPI, false>(a, grid, s);
    }
}

static hipError_t launch_gemm(int variant, int epi, const GemmArgs &a, dim3 grid, hipStream_t s) {
    switch (epi) {
        case EPI_ROWMAJOR: return launch_gemm_v<EPI_ROWMAJOR>(variant, a, grid, s);
        case EPI_RES_IN: return launch_gemm_v<EPI_RES_IN>(variant, a, grid, s);
        case EPI_RES_OUT: return launch_gemm_v<EPI_RES_OUT>(variant, a, grid, s);
        case EPI_SWIGLU: return launch_gemm_v<EPI_SWIGLU>(variant, a, grid, s);
        default: return launch_gemm_v<EPI_PARTIAL>(variant, a, grid, s);
    }
}

// ---------------------------------------------------------------------------------------------- tracing
struct Tracer {
    nexus_ctx *c;
    hipStream_t s;
    bool on;
    TraceRec *rec = nullptr;
    Tracer(nexus_ctx *c_, int phase, int kernel, hipStream_t s_) : c(c_), s(s_) {
        on = c->trace_phase == phase && c->trace_kernel == kernel && c->trace_used < c->trace_pool.size();
        if (on) {
            rec = &c->trace_pool[c->trace_used++];
            (void)hipEventRecord(rec->a, s);
        }
    }
    ~Tracer() {
        if (on) (void)hipEventRecord(rec->b, s);
    }
};

// ---------------------------------------------------------------------------------------------- phase chains
struct PhaseRun {
    nexus_ctx *c;
    int phase;  // NEXUS_PHASE_*
    hipStream_t s;
    int n_xcd;
    int fused_decode = 0;      // > 0: the last fused_decode requests of pb are decode requests (one-token chunks)
    int fused_max_ctx = 0;     // largest context + 1 among them
    int cus;  // CUs the phase's stream may run on
    PhaseWs *ws;  // the phase's workspace (the context's own, or one carved out of the static scratch array)
    int T;
    const nexus_prefill_batch *pb;
    const nexus_decode_batch *db;
    const nexus_kv_cache *kv;
};

// deferred_S (may be null): when given and the GEMM is split along K, the partial slices are left in the workspace
// for the caller's next kernel to sum (see run_rmsnorm_partial) and *deferred_S receives their number, else 0.
static int run_gemm(const PhaseRun &r, int kernel_id, const f16_t *W, int N_packed, const f16_t *X, int K, int epi,
                    void *out, const void *res, const bf16_t *bias, int ld_out, f16_t *out_p32, int out_K,
                    int *deferred_S = nullptr) {
    nexus_ctx *c = r.c;
    PhaseWs &ws = *r.ws;
    const int Kp = p32_kp(K);
    const int n_ftiles = N_packed / 32;
    const GemmPlan p = plan_gemm(r.T, n_ftiles, Kp);
    GemmArgs a{};
    a.W = W, a.X = X, a.n_ftiles = n_ftiles, a.n_ttiles = (r.T + 31) / 32, a.Kp = Kp;
    a.ksteps_per_split = p.ksteps_per_split;
    a.T = r.T, a.N = N_packed;
    a.out = out, a.res = res, a.bias = bias, a.ld_out = ld_out;
    a.out_p32 = out_p32, a.out_Kp = out_p32 ? p32_kp(out_K) : 0;
    a.partial = ws.partial;
    // Ring geometry and tile extent may follow the CU share (they do not change any element's summation order; the
    // split factor S, which does, is problem-only).  Larger tiles move fewer operand bytes through LDS per flop but
    // quantise worse on a given number of CUs.  The choice minimises the sum over the rounds of the grid of the time
    // of one round, which depends on how many CUs the round keeps busy: the chip is power-limited under dense MFMA
    // work and clocks higher when fewer CUs run it.  Fits to measurements on MI355X (the four projections of the 8B-
    // and 70B-shaped layers on 128 ... 256 CUs), microseconds per 4096 elements of K, n = busy CUs: 256 x 256 tiles,
    // one per CU, 72 + 0.14 max(0, n - 128) + 0.21 max(0, n - 192) plus 30 per launch for the fill and the drain of
    // its last round; 256 x 128 tiles, one per CU, 55.5 + 0.06 max(0, n - 128); 128 x 128 tiles, two per CU,
    // 60 + 0.0625 max(0, n - 128), 47 for a last round with at most one tile per CU.  Ties go to the larger tile.
    int variant = p.variant, FS = p.FS, TS = p.TS;
    if (variant == GV_P128 && p.S == 1 && c->allow_p256) {
        const long n128 = (long)((a.n_ttiles + 3) / 4) * ((n_ftiles + 3) / 4);
        const long n256 = (long)((a.n_ttiles + 7) / 8) * ((n_ftiles + 7) / 8);
        const long n256x128 = (long)((a.n_ttiles + 3) / 4) * ((n_ftiles + 7) / 8);
        const double kscale = Kp / 4096.0;
        auto total = [&](long tiles, int per_cu, auto round_us) {
            const long slots = (long)per_cu * r.cus, rem = tiles % slots;
            return kscale * ((double)(tiles / slots) * round_us(r.cus) + (rem ? round_us((int)((rem + per_cu - 1) / per_cu)) : 0.0));
        };
        const double est256 = 30.0 + total(n256, 1, [](int n) { return 72.0 + 0.14 * std::max(0, n - 128) + 0.21 * std::max(0, n - 192); });
        const double est256x128 = total(n256x128, 1, [](int n) { return 55.5 + 0.06 * std::max(0, n - 128); });
        double est128 = total(n128, 2, [](int n) { return 60.0 + 0.0625 * std::max(0, n - 128); });
        if (n128 % (2L * r.cus) && n128 % (2L * r.cus) <= r.cus) est128 -= kscale * 13.0;  // last round: one tile per CU, 47
        // 320 x 256 tiles: the 256 x 256 kernel with five instead of four MFMA tiles per wavefront along the features
        // (1.25x the time per round), where the width divides and the epilogue is the plain one
        double est320 = 1e30;
        if (epi == EPI_ROWMAJOR && n_ftiles % 10 == 0 && (size_t)n_ftiles * Kp * 64 < ((size_t)1 << 32) && (size_t)a.n_ttiles * Kp * 64 < ((size_t)1 << 32))
            est320 = 30.0 + 1.25 * total((long)((a.n_ttiles + 7) / 8) * (n_ftiles / 10), 1,
                                         [](int n) { return 72.0 + 0.14 * std::max(0, n - 128) + 0.21 * std::max(0, n - 192); });
        const double best = std::min(std::min(est256, est256x128), std::min(est128, est320));
        if (c->force_tile ? (c->force_tile == 320 && est320 < 1e30) : est320 == best && est320 < est256) variant = GV_P320, FS = 10, TS = 8;
        else if (c->force_tile ? c->force_tile == 256 : (est256 <= est128 && est256 <= est256x128)) variant = GV_P256, FS = 8, TS = 8;
        else if (c->force_tile ? c->force_tile == 384 : est256x128 <= est128) variant = GV_P256x128, FS = 8, TS = 4;
    }
    // Measured on 64 of the 256 CUs (T = 64): gate/up 113 -> 98 us, down 55 -> 48, O 21.6 -> 18.9 with the wide
    // variant, QKV (too few workgroups left) 27 -> 30; on 96 CUs and more the narrow one wins or ties.
    if (variant == GV_S64 && r.cus <= 64 && (long)((n_ftiles + 7) / 8) * p.S >= 2L * r.cus - r.cus / 4) variant = GV_S64W, FS = 8;
    // 65..128 tokens, measured on config 4's decode batch (128 tokens) on 256 / 96 CUs, 128-feature against 256-feature
    // workgroups: QKV 23 / 44 us against 29 / 46, gate/up 62 / 132 against 80 / 137, O 24 / 37 against 21 / 32, down
    // 45 / 73 against 36 / 61 (the 128 x 128-tile kernel this replaces: 26 / 48, 74 / 147, 23 / 32, 49 / 71).  The
    // wide workgroup wins where the narrow grid would be far more workgroups than the chip has CUs (the deeply split
    // O and down projections); the rule looks at the problem only.
    if (variant == GV_S128 && (long)((n_ftiles + 3) / 4) * p.S > kChipCUs + kChipCUs / 8) variant = GV_S128W, FS = 8;
    const int last_ksteps = Kp / kGemmBK - (p.S - 1) * p.ksteps_per_split;  // the shortest k range of the grid
    if (last_ksteps < kStreamDepth)
        variant = (variant == GV_S64 || variant == GV_S64W) ? (FS = 4, GV_R64)
                  : variant == GV_S32                       ? GV_R32
                  : (variant == GV_S128 || variant == GV_S128W) ? (FS = 4, GV_P128)
                                                            : variant;
    a.n_tblk = (a.n_ttiles + TS - 1) / TS;
    a.n_xcd = r.n_xcd;
    // Tiles resident on one XCD at a time form a 4 x (residents / 4) rectangle instead of a row of token blocks:
    // at 8192 tokens the L2 hit rate of a row is 56% (every tile streams its own token block past the shared weight
    // block), and the rectangle is 7% (256-tiles) to 25% (128-tiles) faster; below ~2048 tokens a row already
    // wraps into a rectangle and the order makes no measurable difference.
    a.group_f = 4;
    const int n_fblk = (n_ftiles + FS - 1) / FS;
    dim3 grid(a.n_tblk * n_fblk, 1, p.S);
    if (p.S > kMaxSlices) return fail(NEXUS_ESTATE, "internal: %d split-K slices, the reductions unroll over %d", p.S, kMaxSlices);
    if (p.S > 1 && (size_t)p.S * r.T * N_packed > ws.partial_elems)
        return fail(NEXUS_ESTATE, "split-K workspace too small (%d x %d x %d)", p.S, r.T, N_packed);
    {
        Tracer tr(c, r.phase, kernel_id, r.s);
        HIP_TRY(launch_gemm(variant, p.S > 1 ? (int)EPI_PARTIAL : epi, a, grid, r.s));
    }
    if (deferred_S) *deferred_S = p.S > 1 ? p.S : 0;
    if (p.S > 1 && !deferred_S) {
        ReduceArgs ra{};
        ra.partial = ws.partial, ra.S = p.S, ra.T = r.T, ra.N = N_packed;
        ra.out = out, ra.res = res, ra.bias = bias, ra.ld_out = ld_out, ra.out_p32 = out_p32, ra.out_Kp = a.out_Kp;
        const size_t n = (size_t)r.T * (N_packed / 4);
        dim3 g((unsigned)((n + 255) / 256));
        Tracer tr(c, r.phase, NEXUS_K_SPLITK_REDUCE, r.s);
        if (epi == EPI_ROWMAJOR) hipLaunchKernelGGL(splitk_reduce_kernel<EPI_ROWMAJOR>, g, dim3(256), 0, r.s, ra);
        else if (epi == EPI_RES_IN) hipLaunchKernelGGL(splitk_reduce_kernel<EPI_RES_IN>, g, dim3(256), 0, r.s, ra);
        else if (epi == EPI_RES_OUT) hipLaunchKernelGGL(splitk_reduce_kernel<EPI_RES_OUT>, g, dim3(256), 0, r.s, ra);
        else hipLaunchKernelGGL(splitk_reduce_kernel<EPI_SWIGLU>, g, dim3(256), 0, r.s, ra);
        HIP_TRY(hipGetLastError());
    }
    return NEXUS_OK;
}

template <int IN>
static int run_rmsnorm(const PhaseRun &r, const void *x, const bf16_t *g, f16_t *out_p32, RmsPartial pp = RmsPartial{}) {
    nexus_ctx *c = r.c;
    const int d = c->m.hidden;
    Tracer tr(c, r.phase, NEXUS_K_RMSNORM, r.s);
    const int Kp = p32_kp(d);
    if (r.T >= 1024) {  // problem-only choice (the two kernels sum the squares in different orders)
        const dim3 grid((r.T + kRmsWaves - 1) / kRmsWaves), block(64 * kRmsWaves);
#define NX_RMS_WAVE(MAXC)                                                                                              \
    {                                                                                                               \
        auto kern = rmsnorm_wave_kernel<MAXC, IN>;                                                                    \
        constexpr int smem = kRmsWaves * (MAXC * 64 + 1) * 16;                                                        \
        static bool done = false;                                                                                   \
        if (!done) {                                                                                                \
            HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem));     \
            done = true;                                                                                            \
        }                                                                                                           \
        hipLaunchKernelGGL(kern, grid, block, smem, r.s, x, g, out_p32, r.T, d, Kp, c->m.rms_eps, pp);              \
    }
        if (d <= 1024) NX_RMS_WAVE(2)
        else if (d <= 2048) NX_RMS_WAVE(4)
        else if (d <= 4096) NX_RMS_WAVE(8)
        else NX_RMS_WAVE(16)
#undef NX_RMS_WAVE
    } else if (d <= 2048) hipLaunchKernelGGL((rmsnorm_kernel<1, IN>), dim3(r.T), dim3(256), 0, r.s, x, g, out_p32, d, Kp, c->m.rms_eps, pp);
    else if (d <= 4096) hipLaunchKernelGGL((rmsnorm_kernel<2, IN>), dim3(r.T), dim3(256), 0, r.s, x, g, out_p32, d, Kp, c->m.rms_eps, pp);
    else hipLaunchKernelGGL((rmsnorm_kernel<4, IN>), dim3(r.T), dim3(256), 0, r.s, x, g, out_p32, d, Kp, c->m.rms_eps, pp);
    HIP_TRY(hipGetLastError());
    return NEXUS_OK;
}

// Key-range splits of the prefill attention: a short chunk has too few (32-token strip, query head) pairs to fill
// the chip's 1024 SIMDs, so its key range is cut into runs handled by separate workgroups.  Problem-only.
static int plan_attn_splits(int n_tokens, int n_q_heads, int max_total_len) {
    const int wave_tasks = ((n_tokens + 31) / 32) * n_q_heads;
    int S = (2048 + wave_tasks / 2) / wave_tasks;
    const int tiles = (max_total_len + kAttnTile - 1) / kAttnTile;
    S = std::min(S, tiles / 8);  // at least 8 key tiles per split
    return std::max(1, std::min(S, kAttnMaxSplits));
}

template <int HD>
static int launch_attn_prefill(const PhaseRun &r, const AttnPrefillArgs &base) {
    nexus_ctx *c = r.c;
    const int G = c->m.n_q_heads / c->m.n_kv_heads;
    AttnPrefillArgs a = base;
#define NX_ATTN_CASE(GG, SPB)                                                                                        \
    case GG: {                                                                                                       \
        auto kern = attn_prefill_kernel<HD, GG, SPB>;                                                                \
        constexpr int smem = attn_stages(GG * SPB) * 4 * kPage * HD * 2 + kAttnMaxPages * 4;                         \
        static bool done = false;                                                                                    \
        if (!done) {                                                                                                 \
            HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem));      \
            done = true;                                                                                             \
        }                                                                                                            \
        a.tiles_per_req = (r.pb->max_chunk + 32 * SPB - 1) / (32 * SPB);                                             \
        if ((long)a.n_reqs * a.tiles_per_req > 65535) return fail(NEXUS_ESHAPE, "prefill attention grid too large (%d requests x %d tiles)", a.n_reqs, a.tiles_per_req); \
        {                                                                                                            \
            Tracer tr(c, r.phase, NEXUS_K_ATTN_PREFILL, r.s);                                                        \
            hipLaunchKernelGGL(kern, dim3(c->m.n_kv_heads, a.n_reqs * a.tiles_per_req, a.n_splits), dim3(64 * GG * SPB), smem, r.s, a); \
        }                                                                                                            \
        HIP_TRY(hipGetLastError());                                                                                  \
        if (a.n_splits > 1) {                                                                                        \
            Tracer tr(c, r.phase, NEXUS_K_ATTN_MERGE, r.s);                                                          \
            hipLaunchKernelGGL((attn_prefill_merge_kernel<HD, SPB>), dim3((r.T - r.fused_decode) * ((c->m.n_q_heads * HD + 511) / 512)), dim3(64), 0, r.s, a); /* decode rows of a fused batch are not this kernel's */ \
        }                                                                                                            \
        break;                                                                                                       \
    }
    switch (G) {
        NX_ATTN_CASE(1, 4)
        NX_ATTN_CASE(2, 2)
        NX_ATTN_CASE(4, 1)
        NX_ATTN_CASE(5, 1)
        NX_ATTN_CASE(8, 1)
        default: return fail(NEXUS_ESHAPE, "query/kv head ratio %d has no prefill attention kernel (1, 2, 4, 5, 8)", G);
    }
#undef NX_ATTN_CASE
    HIP_TRY(hipGetLastError());
    return NEXUS_OK;
}

template <int HD>
static int launch_attn_decode(const PhaseRun &r, const AttnDecodeArgs &a) {
    nexus_ctx *c = r.c;
    const int G = c->m.n_q_heads / c->m.n_kv_heads;
    const int items = a.n_reqs * c->m.n_kv_heads * a.max_spans;
    dim3 grid((items + kDecWaves - 1) / kDecWaves), mgrid(a.n_reqs * c->m.n_q_heads);
#define NX_DEC_CASE(GG)                                                                           \
    case GG: {                                                                                    \
        {                                                                                         \
            Tracer tr(c, r.phase, NEXUS_K_ATTN_DECODE, r.s);                                      \
            hipLaunchKernelGGL((attn_decode_kernel<HD, GG>), grid, dim3(64 * kDecWaves), 0, r.s, a);         \
        }                                                                                         \
        HIP_TRY(hipGetLastError());                                                               \
        {                                                                                         \
            Tracer tr(c, r.phase, NEXUS_K_ATTN_MERGE, r.s);                                       \
            hipLaunchKernelGGL((attn_merge_kernel<HD, GG>), mgrid, dim3(64), 0, r.s, a);          \
        }                                                                                         \
        break;                                                                                    \
    }
    switch (G) {
        NX_DEC_CASE(1)
        NX_DEC_CASE(2)
        NX_DEC_CASE(4)
        NX_DEC_CASE(5)
        NX_DEC_CASE(8)
        default: return fail(NEXUS_ESHAPE, "query/kv head ratio %d has no decode attention kernel (1, 2, 4, 5, 8)", G);
    }
#undef NX_DEC_CASE
    HIP_TRY(hipGetLastError());
    return NEXUS_OK;
}

// down_pending > 0: the previous layer's down projection left that many split-K slices in the workspace and its
// residual in x1; x_in (that layer's output) is still unwritten and this layer's first norm produces it.
// defer_down (may be null): when given and this layer's down projection is split along K, its slices are left for
// the next layer in the same way and *defer_down receives their number, else 0.
static int run_layer(const PhaseRun &r, int layer, const bf16_t *x_in, bf16_t *y_out, int down_pending, int *defer_down) {
    nexus_ctx *c = r.c;
    const nexus_model_desc &m = c->m;
    PhaseWs &ws = *r.ws;
    const LayerW &L = c->layers[layer];
    const bool prefill = r.phase == NEXUS_PHASE_PREFILL;
    bf16_t *k_pool = (bf16_t *)((char *)r.kv->k_pool + (size_t)layer * r.kv->layer_stride_bytes);
    bf16_t *v_pool = (bf16_t *)((char *)r.kv->v_pool + (size_t)layer * r.kv->layer_stride_bytes);

    if (down_pending) {
        RmsPartial pp{ws.partial, down_pending, r.T, nullptr, nullptr, ws.x1, const_cast<bf16_t *>(x_in)};
        NX_TRY(run_rmsnorm<RMS_IN_PARTIAL_Y>(r, nullptr, L.g1, ws.h, pp));
    } else {
        NX_TRY(run_rmsnorm<RMS_IN_BF16>(r, x_in, L.g1, ws.h));
    }
    int qkv_slices = 0;  // a split-K QKV projection is summed by the rotary kernel
    NX_TRY(run_gemm(r, NEXUS_K_GEMM_QKV, L.wqkv, c->n_qkv, ws.h, m.hidden, EPI_ROWMAJOR, ws.qkv, nullptr, L.bqkv, c->n_qkv,
                    nullptr, 0, &qkv_slices));
    {
        RopeArgs a{};
        a.partial = qkv_slices ? ws.partial : nullptr, a.S = qkv_slices, a.bias = L.bqkv;
        a.qkv = ws.qkv, a.T = r.T, a.Hq = m.n_q_heads, a.Hkv = m.n_kv_heads, a.hd = m.head_dim;
        a.rope_tab = c->rope_tab, a.n_pos = c->lim.max_positions;
        a.cu_chunk = prefill ? r.pb->cu_chunk : nullptr;
        a.pos_base = prefill ? r.pb->prefix_len : r.db->ctx_len;
        a.n_reqs = prefill ? r.pb->n_reqs : r.db->n_reqs;
        a.page_table = prefill ? r.pb->page_table : r.db->page_table;
        a.max_pages = prefill ? r.pb->max_pages : r.db->max_pages;
        a.k_pool = k_pool, a.v_pool = v_pool, a.n_pages = r.kv->n_pages, a.q_out = ws.q;
        Tracer tr(c, r.phase, NEXUS_K_ROPE_APPEND, r.s);
        // prefill: 4 groups of 8 rows per 32-row tile of the request-aligned rows (at most T / 32 + n_reqs tiles)
        const int groups = 4 * (r.T / 32 + a.n_reqs);
        const int share = std::max(1, std::min(8, 2048 / groups));  // workgroups per group, so that ~2048 are in the grid
        if (prefill) hipLaunchKernelGGL(rope_append_prefill_kernel, dim3(groups, share), dim3(256), 0, r.s, a);
        else hipLaunchKernelGGL(rope_append_decode_kernel, dim3(r.T, std::max(1, std::min(4, 256 / std::max(1, r.T)))), dim3(256), 0, r.s, a);
        HIP_TRY(hipGetLastError());
    }
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)m.head_dim);
    if (prefill) {
        AttnPrefillArgs a{};
        a.q = ws.q, a.out = ws.attn, a.cu_chunk = r.pb->cu_chunk, a.prefix_len = r.pb->prefix_len, a.page_table = r.pb->page_table;
        a.n_reqs = r.pb->n_reqs - r.fused_decode, a.max_pages = r.pb->max_pages;
        a.k_pool = k_pool, a.v_pool = v_pool, a.n_pages = r.kv->n_pages, a.Hq = m.n_q_heads, a.Hkv = m.n_kv_heads;
        a.scale_log2e = scale_log2e;
        a.n_splits = plan_attn_splits(r.T, m.n_q_heads, r.pb->max_total_len);
        a.part_o = (f16_t *)ws.part_o, a.part_ml = ws.part_ml, a.T = r.T;
        if (a.n_reqs > 0) NX_TRY(m.head_dim == 128 ? launch_attn_prefill<128>(r, a) : launch_attn_prefill<64>(r, a));
        if (r.fused_decode) {
            // the decode requests at the tail of the batch take the decode attention kernel: same queries (prefill
            // layout), same pools (their new K/V was appended by the rotary kernel above), outputs into the same
            // attention buffer; the span partials use the decode phase's workspace
            const int lead = r.pb->n_reqs - r.fused_decode;
            AttnDecodeArgs d{};
            d.q = ws.q, d.ctx_len = r.pb->prefix_len + lead, d.page_table = r.pb->page_table + (size_t)lead * r.pb->max_pages;
            d.n_reqs = r.fused_decode, d.max_pages = r.pb->max_pages, d.max_spans = (r.fused_max_ctx + kSpan - 1) / kSpan;
            d.k_pool = k_pool, d.v_pool = v_pool, d.n_pages = r.kv->n_pages, d.Hq = m.n_q_heads, d.Hkv = m.n_kv_heads;
            d.scale_log2e = scale_log2e, d.part_o = (f16_t *)c->ws[NEXUS_PHASE_DECODE].part_o, d.part_ml = c->ws[NEXUS_PHASE_DECODE].part_ml;
            d.out = ws.attn, d.lead_cu = r.pb->cu_chunk, d.n_lead = lead, d.out_row0 = r.pb->n_tokens - r.fused_decode;
            NX_TRY(m.head_dim == 128 ? launch_attn_decode<128>(r, d) : launch_attn_decode<64>(r, d));
        }
    } else {
        AttnDecodeArgs a{};
        a.q = ws.q, a.ctx_len = r.db->ctx_len, a.page_table = r.db->page_table, a.n_reqs = r.db->n_reqs;
        a.max_pages = r.db->max_pages, a.max_spans = (r.db->max_ctx + kSpan - 1) / kSpan;
        a.k_pool = k_pool, a.v_pool = v_pool, a.n_pages = r.kv->n_pages, a.Hq = m.n_q_heads, a.Hkv = m.n_kv_heads;
        a.scale_log2e = scale_log2e, a.part_o = (f16_t *)ws.part_o, a.part_ml = ws.part_ml, a.out = ws.attn;
        NX_TRY(m.head_dim == 128 ? launch_attn_decode<128>(r, a) : launch_attn_decode<64>(r, a));
    }
    // x1 = x + attn W_o^T, h2 = RMSNorm(x1): when the projection is split along K its reduction, the residual add
    // and the norm are one kernel
    int o_slices = 0;
    NX_TRY(run_gemm(r, NEXUS_K_GEMM_O, L.wo, m.hidden, ws.attn, c->q_dim, EPI_RES_IN, ws.x1, x_in, nullptr, m.hidden,
                    nullptr, 0, &o_slices));
    if (o_slices) {
        RmsPartial pp{ws.partial, o_slices, r.T, (const bf16_t *)x_in, ws.x1, nullptr, nullptr};
        NX_TRY(run_rmsnorm<RMS_IN_PARTIAL>(r, nullptr, L.g2, ws.h, pp));
    } else {
        NX_TRY(run_rmsnorm<RMS_IN_F32>(r, ws.x1, L.g2, ws.h));
    }
    NX_TRY(run_gemm(r, NEXUS_K_GEMM_GATE_UP, L.wgu, 2 * m.ffn, ws.h, m.hidden, EPI_SWIGLU, nullptr, nullptr, nullptr, 0,
                    ws.act, m.ffn));
    NX_TRY(run_gemm(r, NEXUS_K_GEMM_DOWN, L.wdown, m.hidden, ws.act, m.ffn, EPI_RES_OUT, y_out, ws.x1, nullptr, m.hidden,
                    nullptr, 0, defer_down));
    return NEXUS_OK;
}

// A phase's pass over a layer range, enqueued one layer at a time so that the host can alternate between the two
// phases of a step (neither stream then sits idle behind the other phase's launches).
// tail (may be null): layers from tail_from on are launched with *tail -- the same phase, batch and workspace on
// another stream and CU share -- ordered after the layers before them by an event.
struct PhaseCursor {
    PhaseRun r;
    int layer_begin, layer_end, l;
    const PhaseRun *tail = nullptr;
    int tail_from = 0;
    const bf16_t *x;
    int pending = 0;  // split-K slices of the previous layer's down projection, summed by this layer's first norm
    PhaseCursor(const PhaseRun &run, int lb, int le, const PhaseRun *t = nullptr, int from = 0)
        : r(run), layer_begin(lb), layer_end(le), l(lb), tail(t), tail_from(from),
          x((const bf16_t *)(run.phase == NEXUS_PHASE_PREFILL ? run.pb->x : run.db->x)) {}
    bool done() const { return l >= layer_end; }
    hipStream_t last_stream() const { return tail && layer_end > tail_from ? tail->s : r.s; }
    int step() {
        PhaseWs &ws = *r.ws;
        const bool last = l + 1 == layer_end;
        bf16_t *y = last ? (bf16_t *)(r.phase == NEXUS_PHASE_PREFILL ? r.pb->y : r.db->y) : ws.xbuf[(l - layer_begin) & 1];
        int next_pending = 0;
        if (tail && l == tail_from && tail->s != r.s) {
            HIP_TRY(hipEventRecord(r.c->ev_hand, r.s));
            HIP_TRY(hipStreamWaitEvent(tail->s, r.c->ev_hand, 0));
        }
        NX_TRY(run_layer(tail && l >= tail_from ? *tail : r, l, x, y, pending, last ? nullptr : &next_pending));
        pending = next_pending;
        x = y;
        ++l;
        return NEXUS_OK;
    }
};
static int run_phase(const PhaseRun &r, int layer_begin, int layer_end) {
    PhaseCursor pc(r, layer_begin, layer_end);
    while (!pc.done()) NX_TRY(pc.step());
    return NEXUS_OK;
}

// ---------------------------------------------------------------------------------------------- validation
static int check_layers(nexus_ctx *c, int lb, int le) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    if (lb < 0 || le > c->m.n_layers || lb >= le) return fail(NEXUS_EINVAL, "layer range [%d, %d) outside [0, %d)", lb, le, c->m.n_layers);
    for (int l = lb; l < le; ++l)
        if (!c->layers[l].loaded) return fail(NEXUS_ESTATE, "layer %d has no weights loaded", l);
    return NEXUS_OK;
}
static int check_kv(nexus_ctx *c, const nexus_kv_cache *kv, int le) {
    if (!kv || !kv->k_pool || !kv->v_pool) return fail(NEXUS_EINVAL, "null KV cache or pool");
    if (kv->n_pages <= 0) return fail(NEXUS_EINVAL, "n_pages must be positive");
    const int64_t need = (int64_t)kv->n_pages * c->kv_dim * kPage * 2;
    if (le > 1 && kv->layer_stride_bytes < need) return fail(NEXUS_EINVAL, "layer_stride_bytes %lld smaller than one layer's pool (%lld)",
                                                              (long long)kv->layer_stride_bytes, (long long)need);
    if (((uintptr_t)kv->k_pool | (uintptr_t)kv->v_pool | (uintptr_t)kv->layer_stride_bytes) & 15) return fail(NEXUS_EINVAL, "KV pools must be 16-byte aligned");
    return NEXUS_OK;
}
static int check_prefill(nexus_ctx *c, const nexus_prefill_batch *b) {
    if (!b) return fail(NEXUS_EINVAL, "null prefill batch");
    if (!b->x || !b->y || !b->cu_chunk || !b->prefix_len || !b->page_table) return fail(NEXUS_EINVAL, "null pointer in prefill batch");
    if (b->n_reqs <= 0 || b->n_tokens <= 0) return fail(NEXUS_EINVAL, "prefill batch needs n_reqs > 0 and n_tokens > 0");
    if (b->n_reqs > c->lim.max_prefill_reqs || b->n_tokens > c->lim.max_prefill_tokens)
        return fail(NEXUS_ESHAPE, "prefill batch (%d reqs, %d tokens) exceeds context limits (%d, %d)", b->n_reqs, b->n_tokens,
                    c->lim.max_prefill_reqs, c->lim.max_prefill_tokens);
    if (b->max_pages <= 0 || b->max_chunk <= 0 || b->max_chunk > b->n_tokens || b->max_total_len < b->max_chunk)
        return fail(NEXUS_EINVAL, "inconsistent prefill hints (max_pages %d, max_chunk %d, max_total_len %d)", b->max_pages, b->max_chunk,
                    b->max_total_len);
    if (b->max_total_len > c->lim.max_positions) return fail(NEXUS_ESHAPE, "max_total_len %d exceeds max_positions %d", b->max_total_len, c->lim.max_positions);
    if (b->max_total_len > kAttnMaxPages * kPage) return fail(NEXUS_ESHAPE, "max_total_len %d exceeds the %d tokens a prefill workgroup can address", b->max_total_len, kAttnMaxPages * kPage);
    if ((int64_t)b->max_pages * kPage < b->max_total_len) return fail(NEXUS_EINVAL, "page table rows (%d pages) cannot hold max_total_len %d", b->max_pages, b->max_total_len);
    if (((uintptr_t)b->x | (uintptr_t)b->y) & 15) return fail(NEXUS_EINVAL, "x / y must be 16-byte aligned");
    return NEXUS_OK;
}
static int check_decode(nexus_ctx *c, const nexus_decode_batch *b) {
    if (!b) return fail(NEXUS_EINVAL, "null decode batch");
    if (!b->x || !b->y || !b->ctx_len || !b->page_table) return fail(NEXUS_EINVAL, "null pointer in decode batch");
    if (b->n_reqs <= 0) return fail(NEXUS_EINVAL, "decode batch needs n_reqs > 0");
    if (b->n_reqs > c->lim.max_decode_reqs) return fail(NEXUS_ESHAPE, "decode batch of %d exceeds limit %d", b->n_reqs, c->lim.max_decode_reqs);
    if (b->max_pages <= 0 || b->max_ctx <= 0) return fail(NEXUS_EINVAL, "inconsistent decode hints (max_pages %d, max_ctx %d)", b->max_pages, b->max_ctx);
    if (b->max_ctx > c->lim.max_positions) return fail(NEXUS_ESHAPE, "max_ctx %d exceeds max_positions %d", b->max_ctx, c->lim.max_positions);
    if ((int64_t)b->max_pages * kPage < b->max_ctx) return fail(NEXUS_EINVAL, "page table rows (%d pages) cannot hold max_ctx %d", b->max_pages, b->max_ctx);
    if (((uintptr_t)b->x | (uintptr_t)b->y) & 15) return fail(NEXUS_EINVAL, "x / y must be 16-byte aligned");
    return NEXUS_OK;
}

// Debug mode: the device-side integer arrays of a step are copied to the host and validated before anything is
// launched.  The copy runs on the context's own stream and the call waits for it, so the arrays must be complete
// when the step call is made.
static int debug_validate(nexus_ctx *c, const nexus_prefill_batch *pb, const nexus_decode_batch *db, const nexus_kv_cache *kv) {
    if (!c->debug_checks) return NEXUS_OK;
    std::vector<int32_t> cu, pre, ptp, ctx, ptd;
    auto fetch = [&](std::vector<int32_t> &dst, const int32_t *src, size_t n) -> int {
        dst.resize(n);
        if (n) HIP_TRY(hipMemcpyAsync(dst.data(), src, n * sizeof(int32_t), hipMemcpyDeviceToHost, c->s_main));
        return NEXUS_OK;
    };
    if (pb) {
        NX_TRY(fetch(cu, pb->cu_chunk, (size_t)pb->n_reqs + 1));
        NX_TRY(fetch(pre, pb->prefix_len, (size_t)pb->n_reqs));
        NX_TRY(fetch(ptp, pb->page_table, (size_t)pb->n_reqs * pb->max_pages));
    }
    if (db) {
        NX_TRY(fetch(ctx, db->ctx_len, (size_t)db->n_reqs));
        NX_TRY(fetch(ptd, db->page_table, (size_t)db->n_reqs * db->max_pages));
    }
    HIP_TRY(hipStreamSynchronize(c->s_main));
    return nexus_validate_batches(kv->n_pages, kPage, pb ? pb->n_reqs : 0, pb ? pb->n_tokens : 0, cu.data(), pre.data(), ptp.data(),
                                  pb ? pb->max_pages : 0, pb ? pb->max_chunk : 0, pb ? pb->max_total_len : 0, db ? db->n_reqs : 0,
                                  ctx.data(), ptd.data(), db ? db->max_pages : 0, db ? db->max_ctx : 0);
}

// ---------------------------------------------------------------------------------------------- CU masks
// A CU mask is a bit per CU.  On a multi-die part the driver deals consecutive mask bits to the dies round-robin
// (bit i -> die i % n_xcd, CU i / n_xcd); bits_xcd_major switches to the other order (bit i -> die i / cus_per_xcd).
static void set_cu_bit(nexus_ctx *c, std::vector<uint32_t> &mask, int xcd, int cu) {
    const int bit = c->bits_xcd_major ? xcd * c->cus_per_xcd + cu : cu * c->n_xcd + xcd;
    mask[bit >> 5] |= 1u << (bit & 31);
}

static int make_layout(nexus_ctx *c, int p_cus, int d_cus, Layout *out) {
    Layout L;
    L.p_cus = p_cus, L.d_cus = d_cus;
    if (p_cus == 0 && d_cus == 0) {
        HIP_TRY(hipStreamCreateWithFlags(&L.sp, hipStreamNonBlocking));
        L.sd = L.sp;
        L.p_xcd = L.d_xcd = c->n_xcd;
        *out = L;
        return NEXUS_OK;
    }
    const int words = (c->n_cus + 31) / 32;
    std::vector<uint32_t> mp(words, 0), md(words, 0);
    // Every XCD gives each phase the same number of its CUs.  This is the only workable topology: the driver
    // rejects a queue mask that leaves an XCD without CUs, and workgroups are dealt to the XCDs round-robin
    // whatever the mask, so unequal per-XCD shares would only unbalance the phase.
    const int pu = p_cus / c->n_xcd, du = d_cus / c->n_xcd;
    for (int x = 0; x < c->n_xcd; ++x) {
        for (int u = 0; u < pu; ++u) set_cu_bit(c, mp, x, u);
        for (int u = c->cus_per_xcd - du; u < c->cus_per_xcd; ++u) set_cu_bit(c, md, x, u);
    }
    L.p_xcd = L.d_xcd = c->n_xcd;
    for (int i = 0; i < words; ++i)
        if (mp[i] & md[i]) return fail(NEXUS_ESTATE, "internal: CU masks overlap");
    HIP_TRY(hipExtStreamCreateWithCUMask(&L.sp, words, mp.data()));
    HIP_TRY(hipExtStreamCreateWithCUMask(&L.sd, words, md.data()));
    *out = L;
    return NEXUS_OK;
}

// A layout about to be destroyed takes its phase-time measurements with it (a later layout may get its address).
static void forget_handover_history(nexus_ctx *c, const Layout *L) {
    if (c->ho_layout == L) c->ho_layout = nullptr;
    for (auto &hs : c->ho_sample)
        if (hs.layout == L) hs.pending = false, hs.layout = nullptr;
}

static void destroy_layout(Layout &L) {
    if (L.sd && L.sd != L.sp) (void)hipStreamDestroy(L.sd);
    if (L.sp) (void)hipStreamDestroy(L.sp);
    L.sp = L.sd = nullptr;
}

// ---------------------------------------------------------------------------------------------- C ABI
extern "C" {

int nexus_debug_token_order(int b, int n) {
    if (n <= 0 || b < 0 || b >= n) return fail(NEXUS_EINVAL, "token order: index %d outside [0, %d)", b, n);
    return xcd_run_index(b, n);
}

int nexus_cu_count(nexus_ctx *c) { return c ? c->n_cus : fail(NEXUS_EINVAL, "null context"); }

int nexus_set_debug_checks(nexus_ctx *c, int on) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    c->debug_checks = on != 0;
    return NEXUS_OK;
}

void nexus_destroy(nexus_ctx *c) {
    if (!c) return;
    DeviceGuard dg(c->device);
    (void)hipDeviceSynchronize();
    for (auto &kv : c->layouts) destroy_layout(kv.second);
    if (c->s_main) (void)hipStreamDestroy(c->s_main);
    for (auto &L : c->layers) {
        (void)hipFree(L.g1), (void)hipFree(L.g2), (void)hipFree(L.wqkv), (void)hipFree(L.bqkv), (void)hipFree(L.wo), (void)hipFree(L.wgu),
            (void)hipFree(L.wdown);
    }
    for (auto &w : c->ws) {
        (void)hipFree(w.h), (void)hipFree(w.qkv), (void)hipFree(w.q), (void)hipFree(w.attn), (void)hipFree(w.x1), (void)hipFree(w.act);
        (void)hipFree(w.xbuf[0]), (void)hipFree(w.xbuf[1]), (void)hipFree(w.partial), (void)hipFree(w.part_o), (void)hipFree(w.part_ml);
    }
    (void)hipFree(c->rope_tab);
    (void)hipFree(c->probe_counts);
    for (auto &hs : c->ho_sample)
        for (hipEvent_t e : {hs.p0, hs.d0, hs.ph, hs.d1})
            if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : {c->ev_fork, c->ev_caller, c->ev_sp0, c->ev_sp1, c->ev_sd0, c->ev_hand, c->ev_ph0[0], c->ev_ph0[1], c->ev_ph1[0], c->ev_ph1[1]})
        if (e) (void)hipEventDestroy(e);
    for (auto &t : c->trace_pool) (void)hipEventDestroy(t.a), (void)hipEventDestroy(t.b);
    delete c;
}

static int alloc_phase_ws(nexus_ctx *c, int phase, int maxT, int max_reqs) {
    const nexus_model_desc &m = c->m;
    PhaseWs &w = c->ws[phase];
    w.maxT = maxT;
    const int Tp = round_up(maxT, 32);
    NX_TRY(dev_alloc(&w.h, p32_elems(Tp, m.hidden), true));
    NX_TRY(dev_alloc(&w.qkv, (size_t)maxT * c->n_qkv, true));
    if (phase == NEXUS_PHASE_PREFILL) {
        w.q_rows = Tp + 32 * max_reqs;
        NX_TRY(dev_alloc(&w.q, p32_elems(w.q_rows, c->q_dim), true));
        size_t items = 0;  // split results of the attention: worst case over the token counts the phase may see
        for (int T = 1; T <= maxT; ++T) {
            const int S = plan_attn_splits(T, m.n_q_heads, c->lim.max_positions);
            if (S > 1) items = std::max(items, (size_t)S * T * m.n_q_heads);
        }
        NX_TRY(dev_alloc(&w.part_o, (items * m.head_dim + 1) / 2, false));  // half elements
        NX_TRY(dev_alloc(&w.part_ml, items * 2, false));
    } else {
        NX_TRY(dev_alloc(&w.q, (size_t)maxT * c->q_dim, true));
        w.max_spans = (c->lim.max_positions + kSpan - 1) / kSpan;
        const int G = m.n_q_heads / m.n_kv_heads;
        const size_t items = (size_t)maxT * m.n_kv_heads * w.max_spans * G;
        NX_TRY(dev_alloc(&w.part_o, (items * m.head_dim + 1) / 2, false));  // half elements
        NX_TRY(dev_alloc(&w.part_ml, items * 2, false));
    }
    NX_TRY(dev_alloc(&w.attn, p32_elems(Tp, c->q_dim), true));
    NX_TRY(dev_alloc(&w.x1, (size_t)maxT * m.hidden, true));
    NX_TRY(dev_alloc(&w.act, p32_elems(Tp, m.ffn), true));
    if (m.n_layers > 1) {
        NX_TRY(dev_alloc(&w.xbuf[0], (size_t)maxT * m.hidden, true));
        NX_TRY(dev_alloc(&w.xbuf[1], (size_t)maxT * m.hidden, true));
    }
    size_t pe = 0;
    const int shapes[4][2] = {{c->n_qkv, m.hidden}, {m.hidden, c->q_dim}, {2 * m.ffn, m.hidden}, {m.hidden, m.ffn}};
    for (auto &s : shapes)  // the split count depends on T, so take the worst case over every T the phase may see
        for (int T = 1; T <= maxT; ++T) {
            const GemmPlan p = plan_gemm(T, s[0] / 32, p32_kp(s[1]));
            if (p.S > 1) pe = std::max(pe, (size_t)p.S * T * s[0]);
        }
    w.partial_elems = pe;
    NX_TRY(dev_alloc(&w.partial, pe, false));
    return NEXUS_OK;
}

int nexus_create(const nexus_model_desc *desc, const nexus_limits *limits, int device, nexus_ctx **out) {
    if (!desc || !limits || !out) return fail(NEXUS_EINVAL, "null argument");
    *out = nullptr;
    const nexus_model_desc &m = *desc;
    if (m.hidden <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.ffn <= 0 || m.n_layers <= 0) return fail(NEXUS_EINVAL, "non-positive model dimension");
    if (m.head_dim != 64 && m.head_dim != 128) return fail(NEXUS_ESHAPE, "head_dim %d not supported (64 or 128)", m.head_dim);
    if (m.page_size != kPage) return fail(NEXUS_ESHAPE, "page_size %d not supported (16)", m.page_size);
    if (m.n_q_heads % m.n_kv_heads) return fail(NEXUS_ESHAPE, "n_q_heads %d not a multiple of n_kv_heads %d", m.n_q_heads, m.n_kv_heads);
    const int G = m.n_q_heads / m.n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 5 && G != 8) return fail(NEXUS_ESHAPE, "query/kv head ratio %d not supported (1, 2, 4, 5, 8)", G);
    if (m.hidden % 32 || m.ffn % 32) return fail(NEXUS_ESHAPE, "hidden and ffn must be multiples of 32");
    if (m.hidden > 8192) return fail(NEXUS_ESHAPE, "hidden %d above 8192", m.hidden);
    if (!(m.rms_eps >= 0.f) || !(m.rope_theta > 0.f)) return fail(NEXUS_EINVAL, "bad rms_eps / rope_theta");
    if (limits->max_prefill_tokens <= 0 || limits->max_prefill_reqs <= 0 || limits->max_decode_reqs <= 0 || limits->max_positions <= 0)
        return fail(NEXUS_EINVAL, "limits must be positive");
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return fail(NEXUS_EINVAL, "device %d outside [0, %d)", device, ndev);

    nexus_ctx *c = new (std::nothrow) nexus_ctx();
    if (!c) return fail(NEXUS_ENOMEM, "out of host memory");
    c->m = m, c->lim = *limits, c->device = device;
    c->q_dim = m.n_q_heads * m.head_dim, c->kv_dim = m.n_kv_heads * m.head_dim, c->n_qkv = c->q_dim + 2 * c->kv_dim;
    c->layers.resize(m.n_layers);
    DeviceGuard dg(device);
    int rc = NEXUS_OK;
    do {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, device) != hipSuccess) { rc = fail(NEXUS_EHIP, "hipGetDeviceProperties failed"); break; }
        c->n_cus = prop.multiProcessorCount;
        c->n_xcd = 8;
        if (c->n_cus % c->n_xcd) c->n_xcd = 1;
        c->cus_per_xcd = c->n_cus / c->n_xcd;
        const char *order = getenv("NEXUS_CU_BIT_ORDER");
        c->bits_xcd_major = order && !strcmp(order, "xcd_major");
        // test hook: one GEMM tile shape for every prefill projection ("128", "256", "256x128"; "320" where it applies), to compare the shapes
        // bit for bit and to time them against each other
        const char *tiles = getenv("NEXUS_GEMM_TILES");
        c->allow_p256 = !(tiles && !strcmp(tiles, "128"));
        c->force_tile = tiles && !strcmp(tiles, "256") ? 256 : tiles && !strcmp(tiles, "256x128") ? 384 : tiles && !strcmp(tiles, "128") ? 128
                        : tiles && !strcmp(tiles, "320") ? 320 : 0;
        if (const char *dbg = getenv("NEXUS_DEBUG_CHECKS")) c->debug_checks = atoi(dbg) != 0;
        if (const char *ml = getenv("NEXUS_MAX_LAYOUTS")) c->max_layouts = std::max(1, std::min(64, atoi(ml)));
        if (hipStreamCreateWithFlags(&c->s_main, hipStreamNonBlocking) != hipSuccess) { rc = fail(NEXUS_EHIP, "stream creation failed"); break; }
        for (hipEvent_t *e : {&c->ev_fork, &c->ev_caller, &c->ev_sp0, &c->ev_sp1, &c->ev_sd0, &c->ev_hand, &c->ev_ph0[0], &c->ev_ph0[1], &c->ev_ph1[0], &c->ev_ph1[1]})
            if (hipEventCreateWithFlags(e, hipEventDisableSystemFence) != hipSuccess) { rc = fail(NEXUS_EHIP, "event creation failed"); break; }
        for (auto &hs : c->ho_sample)
            for (hipEvent_t *e : {&hs.p0, &hs.d0, &hs.ph, &hs.d1})
                if (hipEventCreate(e) != hipSuccess) { rc = fail(NEXUS_EHIP, "event creation failed"); break; }
        if (rc) break;
        if ((rc = alloc_phase_ws(c, NEXUS_PHASE_PREFILL, limits->max_prefill_tokens, limits->max_prefill_reqs))) break;
        if ((rc = alloc_phase_ws(c, NEXUS_PHASE_DECODE, limits->max_decode_reqs, limits->max_decode_reqs))) break;
        const int half = m.head_dim / 2;
        if ((rc = dev_alloc(&c->rope_tab, (size_t)limits->max_positions * half, false))) break;
        if ((rc = dev_alloc(&c->probe_counts, 8 * 128, true))) break;
        if ((rc = scratch_address(device, &c->scratch_dev))) break;
        const size_t n = (size_t)limits->max_positions * half;
        hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->s_main, c->rope_tab, limits->max_positions, half,
                           (double)m.rope_theta);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(c->s_main) != hipSuccess) { rc = fail(NEXUS_EHIP, "rotary table kernel failed"); break; }
        Layout L;
        if ((rc = make_layout(c, 0, 0, &L))) break;
        c->layouts[0] = L;
        c->cur = &c->layouts[0];
    } while (0);
    if (rc) {
        nexus_destroy(c);
        return rc;
    }
    *out = c;
    return NEXUS_OK;
}

int nexus_sync(nexus_ctx *c) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    DeviceGuard dg(c->device);
    HIP_TRY(hipStreamSynchronize(c->s_main));
    for (auto &kv : c->layouts) {
        HIP_TRY(hipStreamSynchronize(kv.second.sp));
        if (kv.second.sd != kv.second.sp) HIP_TRY(hipStreamSynchronize(kv.second.sd));
    }
    return NEXUS_OK;
}

static int pack_one(nexus_ctx *c, const void *src, int N, int K, int interleave_F, f16_t **dst) {
    const int Kp = p32_kp(K), Np = round_up(N, 32);
    if (!*dst) NX_TRY(dev_alloc(dst, (size_t)Np * Kp, false));
    const size_t n = (size_t)Np * (Kp / 8);
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->s_main, (const bf16_t *)src, *dst, N, K, Kp,
                       interleave_F);
    HIP_TRY(hipGetLastError());
    return NEXUS_OK;
}

int nexus_load_layer(nexus_ctx *c, int layer, const nexus_layer_weights *w) {
    if (!c || !w) return fail(NEXUS_EINVAL, "null argument");
    if (layer < 0 || layer >= c->m.n_layers) return fail(NEXUS_EINVAL, "layer %d outside [0, %d)", layer, c->m.n_layers);
    if (!w->attn_norm_g || !w->w_qkv || !w->w_o || !w->ffn_norm_g || !w->w_gate_up || !w->w_down) return fail(NEXUS_EINVAL, "null weight pointer");
    DeviceGuard dg(c->device);
    const nexus_model_desc &m = c->m;
    LayerW &L = c->layers[layer];
    L.loaded = false;
    if (!L.g1) NX_TRY(dev_alloc(&L.g1, m.hidden, false));
    if (!L.g2) NX_TRY(dev_alloc(&L.g2, m.hidden, false));
    HIP_TRY(hipMemcpyAsync(L.g1, w->attn_norm_g, (size_t)m.hidden * 2, hipMemcpyDeviceToDevice, c->s_main));
    HIP_TRY(hipMemcpyAsync(L.g2, w->ffn_norm_g, (size_t)m.hidden * 2, hipMemcpyDeviceToDevice, c->s_main));
    if (w->b_qkv) {
        if (!L.bqkv) NX_TRY(dev_alloc(&L.bqkv, c->n_qkv, false));
        HIP_TRY(hipMemcpyAsync(L.bqkv, w->b_qkv, (size_t)c->n_qkv * 2, hipMemcpyDeviceToDevice, c->s_main));
    } else if (L.bqkv) {
        (void)hipFree(L.bqkv);
        L.bqkv = nullptr;
    }
    NX_TRY(pack_one(c, w->w_qkv, c->n_qkv, m.hidden, 0, &L.wqkv));
    NX_TRY(pack_one(c, w->w_o, m.hidden, c->q_dim, 0, &L.wo));
    NX_TRY(pack_one(c, w->w_gate_up, 2 * m.ffn, m.hidden, m.ffn, &L.wgu));
    NX_TRY(pack_one(c, w->w_down, m.hidden, m.ffn, 0, &L.wdown));
    HIP_TRY(hipStreamSynchronize(c->s_main));
    L.loaded = true;
    return NEXUS_OK;
}

static int kv_convert(nexus_ctx *c, const nexus_kv_cache *kv, int layer, void *k_canon, void *v_canon, int32_t page_begin, int32_t page_count,
                      bool import) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    NX_TRY(check_kv(c, kv, layer + 1));
    if (!k_canon || !v_canon) return fail(NEXUS_EINVAL, "null canonical buffer");
    if (layer < 0 || layer >= c->m.n_layers) return fail(NEXUS_EINVAL, "layer %d outside [0, %d)", layer, c->m.n_layers);
    if (page_begin < 0 || page_count < 0 || (int64_t)page_begin + page_count > kv->n_pages) return fail(NEXUS_EINVAL, "page range [%d, +%d) outside the pool of %d", page_begin, page_count, kv->n_pages);
    if (page_count == 0) return NEXUS_OK;
    DeviceGuard dg(c->device);
    const size_t blk = (size_t)kPage * c->m.head_dim;
    const size_t off = (size_t)page_begin * c->m.n_kv_heads * blk;
    bf16_t *kp = (bf16_t *)((char *)kv->k_pool + (size_t)layer * kv->layer_stride_bytes) + off;
    bf16_t *vp = (bf16_t *)((char *)kv->v_pool + (size_t)layer * kv->layer_stride_bytes) + off;
    const int n_blocks = page_count * c->m.n_kv_heads;
    const size_t n = (size_t)n_blocks * blk;
    dim3 grid((unsigned)((n + 255) / 256));
    if (import) hipLaunchKernelGGL(kv_convert_kernel<true>, grid, dim3(256), 0, c->s_main, kp, vp, (bf16_t *)k_canon, (bf16_t *)v_canon, n_blocks, c->m.head_dim);
    else hipLaunchKernelGGL(kv_convert_kernel<false>, grid, dim3(256), 0, c->s_main, kp, vp, (bf16_t *)k_canon, (bf16_t *)v_canon, n_blocks, c->m.head_dim);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(c->s_main));
    return NEXUS_OK;
}

int nexus_kv_import(nexus_ctx *c, const nexus_kv_cache *kv, int layer, const void *k_canon, const void *v_canon, int32_t page_begin,
                    int32_t page_count) {
    return kv_convert(c, kv, layer, (void *)k_canon, (void *)v_canon, page_begin, page_count, true);
}
int nexus_kv_export(nexus_ctx *c, const nexus_kv_cache *kv, int layer, void *k_canon, void *v_canon, int32_t page_begin, int32_t page_count) {
    return kv_convert(c, kv, layer, k_canon, v_canon, page_begin, page_count, false);
}

// Finds the layout of a split, creating its stream pair if it does not exist yet (about 10 ms, once).
static int get_layout(nexus_ctx *c, int prefill_cus, int decode_cus, Layout **out) {
    long key = 0;
    if (prefill_cus == NEXUS_CUS_ALL && decode_cus == NEXUS_CUS_ALL) {
        prefill_cus = decode_cus = 0;
    } else {
        const int gran = c->n_xcd;
        if (prefill_cus <= 0 || decode_cus <= 0) return fail(NEXUS_EINVAL, "CU shares must be positive (or both NEXUS_CUS_ALL)");
        if (prefill_cus % gran || decode_cus % gran) return fail(NEXUS_EINVAL, "CU shares must be multiples of %d (one CU in each XCD)", gran);
        if (prefill_cus + decode_cus > c->n_cus) return fail(NEXUS_EINVAL, "CU shares %d + %d exceed the device's %d CUs", prefill_cus, decode_cus, c->n_cus);
        key = ((long)prefill_cus << 20) | decode_cus;
    }
    auto it = c->layouts.find(key);
    if (it == c->layouts.end()) {
        // Every CU-masked stream owns a hardware queue: keep at most max_layouts partitioned pairs alive and
        // retire the least recently used one (never the current one) before creating another.
        int masked = 0;
        for (auto &kv : c->layouts) masked += kv.first != 0;
        while (masked >= c->max_layouts) {
            auto victim = c->layouts.end();
            for (auto jt = c->layouts.begin(); jt != c->layouts.end(); ++jt)
                if (jt->first != 0 && (c->max_layouts == 1 || &jt->second != c->cur) &&
                    (victim == c->layouts.end() || jt->second.last_use < victim->second.last_use))
                    victim = jt;
            if (victim == c->layouts.end()) break;
            HIP_TRY(hipStreamSynchronize(victim->second.sp));
            HIP_TRY(hipStreamSynchronize(victim->second.sd));
            for (int ph = 0; ph < 2; ++ph)  // its work is complete; a new stream may reuse the handle value
                if (c->done_stream[ph] == victim->second.sp || c->done_stream[ph] == victim->second.sd) c->done_stream[ph] = nullptr;
            if (c->cur == &victim->second) c->cur = &c->layouts[0];
            forget_handover_history(c, &victim->second);
            destroy_layout(victim->second);
            c->layouts.erase(victim);
            --masked;
        }
        Layout L;
        NX_TRY(make_layout(c, prefill_cus, decode_cus, &L));
        it = c->layouts.emplace(key, L).first;
    }
    it->second.last_use = ++c->use_clock;
    *out = &it->second;
    return NEXUS_OK;
}

int nexus_set_cu_split(nexus_ctx *c, int prefill_cus, int decode_cus) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    DeviceGuard dg(c->device);
    Layout *L = nullptr;
    NX_TRY(get_layout(c, prefill_cus, decode_cus, &L));
    c->cur = L;  // work in flight on the previous layout keeps running there; later launches are ordered after it by events
    return NEXUS_OK;
}

int nexus_prepare_cu_splits(nexus_ctx *c, int n, const int32_t *prefill_cus, const int32_t *decode_cus) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    if (n < 0 || (n > 0 && (!prefill_cus || !decode_cus))) return fail(NEXUS_EINVAL, "bad split list");
    int distinct = 0;
    for (int i = 0; i < n; ++i) distinct += !(prefill_cus[i] == NEXUS_CUS_ALL && decode_cus[i] == NEXUS_CUS_ALL);
    if (distinct > c->max_layouts) return fail(NEXUS_ESHAPE, "%d partitioned layouts asked for, at most %d are kept alive", distinct, c->max_layouts);
    DeviceGuard dg(c->device);
    for (int i = 0; i < n; ++i) {
        Layout *L = nullptr;
        NX_TRY(get_layout(c, prefill_cus[i], decode_cus[i], &L));
    }
    return NEXUS_OK;
}

int nexus_retire_cu_splits(nexus_ctx *c) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    DeviceGuard dg(c->device);
    for (auto it = c->layouts.begin(); it != c->layouts.end();) {
        if (it->first == 0 || &it->second == c->cur) {
            ++it;
            continue;
        }
        HIP_TRY(hipStreamSynchronize(it->second.sp));
        HIP_TRY(hipStreamSynchronize(it->second.sd));
        for (int ph = 0; ph < 2; ++ph)  // its work is complete; a new stream may reuse the handle value
            if (c->done_stream[ph] == it->second.sp || c->done_stream[ph] == it->second.sd) c->done_stream[ph] = nullptr;
        forget_handover_history(c, &it->second);
        destroy_layout(it->second);
        it = c->layouts.erase(it);
    }
    return NEXUS_OK;
}

static PhaseRun make_run(nexus_ctx *c, int phase, const nexus_prefill_batch *pb, const nexus_decode_batch *db, const nexus_kv_cache *kv) {
    PhaseRun r{};
    r.c = c, r.phase = phase, r.pb = pb, r.db = db, r.kv = kv;
    r.s = phase == NEXUS_PHASE_PREFILL ? c->cur->sp : c->cur->sd;
    r.n_xcd = phase == NEXUS_PHASE_PREFILL ? c->cur->p_xcd : c->cur->d_xcd;
    r.cus = phase == NEXUS_PHASE_PREFILL ? c->cur->p_cus : c->cur->d_cus;
    if (r.cus <= 0) r.cus = c->n_cus;
    r.ws = &c->ws[phase];
    r.T = phase == NEXUS_PHASE_PREFILL ? pb->n_tokens : db->n_reqs;
    return r;
}

// Orders stream s after the last launch that used `phase`'s workspace when that ran on another stream (another
// layout, or the other stream of this one); on the same stream the stream's own order does it.
static int order_after(nexus_ctx *c, hipStream_t s, int phase) {
    if (c->ph_recorded[phase] && c->done_stream[phase] != s) HIP_TRY(hipStreamWaitEvent(s, c->ev_ph1[phase], 0));
    return NEXUS_OK;
}
static int mark_done(nexus_ctx *c, hipStream_t s, int phase, bool timed) {
    HIP_TRY(hipEventRecord(c->ev_ph1[phase], s));
    c->ph_recorded[phase] = true, c->ph_timed[phase] = timed, c->done_stream[phase] = s;
    return NEXUS_OK;
}

// A phase on its own: bracketed by events on the phase's stream so that the caller can poll for its completion
// and read its duration while the other phase keeps running.  It follows the previous launch of the same phase
// (and, for the fused step, which borrows the decode phase's attention workspace, of the decode phase too), never
// the other phase: the two phase loops stay independent.
static int run_single_phase(nexus_ctx *c, const PhaseRun &r, int lb, int le) {
    NX_TRY(order_after(c, r.s, r.phase));
    if (r.fused_decode) NX_TRY(order_after(c, r.s, NEXUS_PHASE_DECODE));
    HIP_TRY(hipEventRecord(c->ev_ph0[r.phase], r.s));
    NX_TRY(run_phase(r, lb, le));
    NX_TRY(mark_done(c, r.s, r.phase, true));
    if (r.fused_decode) NX_TRY(mark_done(c, r.s, NEXUS_PHASE_DECODE, false));
    return NEXUS_OK;
}

int nexus_prefill_chunk(nexus_ctx *c, int lb, int le, const nexus_prefill_batch *pb, const nexus_kv_cache *kv) {
    NX_TRY(check_layers(c, lb, le));
    NX_TRY(check_kv(c, kv, le));
    NX_TRY(check_prefill(c, pb));
    DeviceGuard dg(c->device);
    NX_TRY(debug_validate(c, pb, nullptr, kv));
    return run_single_phase(c, make_run(c, NEXUS_PHASE_PREFILL, pb, nullptr, kv), lb, le);
}

int nexus_decode_step(nexus_ctx *c, int lb, int le, const nexus_decode_batch *db, const nexus_kv_cache *kv) {
    NX_TRY(check_layers(c, lb, le));
    NX_TRY(check_kv(c, kv, le));
    NX_TRY(check_decode(c, db));
    DeviceGuard dg(c->device);
    NX_TRY(debug_validate(c, nullptr, db, kv));
    return run_single_phase(c, make_run(c, NEXUS_PHASE_DECODE, nullptr, db, kv), lb, le);
}

// Lays the decode phase's workspace for T requests with contexts of at most max_ctx positions out over `base`
// (256-byte aligned pieces).  Returns the bytes needed; *zero_bytes is the leading part that must be cleared before
// use (tile-ordered operands whose padding the GEMMs read, and everything a previous call of another shape may have
// left behind).  With base == nullptr it only measures.
static size_t carve_decode_ws(const nexus_ctx *c, int T, int max_ctx, bool multi_layer, unsigned char *base, PhaseWs *w, size_t *zero_bytes) {
    const nexus_model_desc &m = c->m;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        unsigned char *p = base ? base + off : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    const int Tp = round_up(T, 32);
    PhaseWs ws{};
    ws.maxT = T;
    ws.h = (f16_t *)take(p32_elems(Tp, m.hidden) * 2);
    ws.attn = (f16_t *)take(p32_elems(Tp, c->q_dim) * 2);
    ws.act = (f16_t *)take(p32_elems(Tp, m.ffn) * 2);
    ws.qkv = (f16_t *)take((size_t)T * c->n_qkv * 2);
    ws.q = (bf16_t *)take((size_t)T * c->q_dim * 2);
    ws.x1 = (float *)take((size_t)T * m.hidden * 4);
    if (multi_layer) {
        ws.xbuf[0] = (bf16_t *)take((size_t)T * m.hidden * 2);
        ws.xbuf[1] = (bf16_t *)take((size_t)T * m.hidden * 2);
    }
    *zero_bytes = off;
    ws.max_spans = (max_ctx + kSpan - 1) / kSpan;
    const size_t items = (size_t)T * m.n_q_heads * ws.max_spans;  // (request, kv head, span) x the G heads of the kv head
    ws.part_o = (float *)take(items * m.head_dim * 2);  // half elements
    ws.part_ml = (float *)take(items * 2 * 4);
    size_t pe = 0;
    const int shapes[4][2] = {{c->n_qkv, m.hidden}, {m.hidden, c->q_dim}, {2 * m.ffn, m.hidden}, {m.hidden, m.ffn}};
    for (auto &sh : shapes) {
        const GemmPlan p = plan_gemm(T, sh[0] / 32, p32_kp(sh[1]));
        if (p.S > 1) pe = std::max(pe, (size_t)p.S * T * sh[0]);
    }
    ws.partial_elems = pe;
    ws.partial = (float *)take(pe * 4);
    if (w) *w = ws;
    return off;
}

int nexus_decode_step_noalloc(nexus_ctx *c, int lb, int le, const nexus_decode_batch *db, const nexus_kv_cache *kv) {
    NX_TRY(check_layers(c, lb, le));
    NX_TRY(check_kv(c, kv, le));
    NX_TRY(check_decode(c, db));
    PhaseWs ws;
    size_t zero_bytes = 0;
    const size_t need = carve_decode_ws(c, db->n_reqs, db->max_ctx, le - lb > 1, nullptr, nullptr, &zero_bytes);
    if (need > kScratchBytes)
        return fail(NEXUS_ESHAPE, "a decode step of %d requests with contexts up to %d needs %zu bytes of workspace, the static scratch array holds %zu",
                    db->n_reqs, db->max_ctx, need, kScratchBytes);
    DeviceGuard dg(c->device);
    NX_TRY(debug_validate(c, nullptr, db, kv));
    unsigned char *base = nullptr;
    NX_TRY(scratch_address(c->device, &base));
    carve_decode_ws(c, db->n_reqs, db->max_ctx, le - lb > 1, base, &ws, &zero_bytes);
    PhaseRun r = make_run(c, NEXUS_PHASE_DECODE, nullptr, db, kv);
    r.ws = &ws;  // only read while the launches below are enqueued
    NX_TRY(order_after(c, r.s, NEXUS_PHASE_DECODE));
    HIP_TRY(hipEventRecord(c->ev_ph0[NEXUS_PHASE_DECODE], r.s));
    const size_t n16 = zero_bytes / 16;  // every piece is a multiple of 256 bytes
    hipLaunchKernelGGL(scratch_clear_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, r.s, (uint4 *)base, n16);
    HIP_TRY(hipGetLastError());
    NX_TRY(run_phase(r, lb, le));
    NX_TRY(mark_done(c, r.s, NEXUS_PHASE_DECODE, true));
    return NEXUS_OK;
}

int nexus_fused_step(nexus_ctx *c, int lb, int le, const nexus_prefill_batch *batch, int32_t n_decode_reqs, int32_t max_decode_ctx,
                     const nexus_kv_cache *kv) {
    NX_TRY(check_layers(c, lb, le));
    NX_TRY(check_kv(c, kv, le));
    NX_TRY(check_prefill(c, batch));
    if (n_decode_reqs < 0 || n_decode_reqs > batch->n_reqs) return fail(NEXUS_EINVAL, "%d decode requests in a batch of %d", n_decode_reqs, batch->n_reqs);
    if (n_decode_reqs > c->lim.max_decode_reqs) return fail(NEXUS_ESHAPE, "%d decode requests exceed limit %d", n_decode_reqs, c->lim.max_decode_reqs);
    if (n_decode_reqs > 0 && (max_decode_ctx <= 0 || max_decode_ctx > c->lim.max_positions || max_decode_ctx > batch->max_total_len))
        return fail(NEXUS_EINVAL, "max_decode_ctx %d outside (0, min(max_positions %d, max_total_len %d)]", max_decode_ctx, c->lim.max_positions, batch->max_total_len);
    if ((int64_t)batch->max_pages * kPage < max_decode_ctx) return fail(NEXUS_EINVAL, "page table rows (%d pages) cannot hold max_decode_ctx %d", batch->max_pages, max_decode_ctx);
    DeviceGuard dg(c->device);
    NX_TRY(debug_validate(c, batch, nullptr, kv));
    PhaseRun r = make_run(c, NEXUS_PHASE_PREFILL, batch, nullptr, kv);
    r.fused_decode = n_decode_reqs, r.fused_max_ctx = max_decode_ctx;
    return run_single_phase(c, r, lb, le);
}

int nexus_phase_query(nexus_ctx *c, int phase) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    if (phase != NEXUS_PHASE_PREFILL && phase != NEXUS_PHASE_DECODE) return fail(NEXUS_EINVAL, "unknown phase %d", phase);
    if (!c->ph_recorded[phase]) return 1;
    DeviceGuard dg(c->device);
    const hipError_t e = hipEventQuery(c->ev_ph1[phase]);
    if (e == hipSuccess) return 1;
    if (e == hipErrorNotReady) return 0;
    return fail(NEXUS_EHIP, "hipEventQuery failed: %s", hipGetErrorString(e));
}

int nexus_phase_wait(nexus_ctx *c, int phase, float *elapsed_ms) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    if (phase != NEXUS_PHASE_PREFILL && phase != NEXUS_PHASE_DECODE) return fail(NEXUS_EINVAL, "unknown phase %d", phase);
    if (!c->ph_recorded[phase]) return fail(NEXUS_ESTATE, "nothing has been launched for this phase");
    DeviceGuard dg(c->device);
    HIP_TRY(hipEventSynchronize(c->ev_ph1[phase]));
    if (elapsed_ms) {
        if (c->ph_timed[phase]) HIP_TRY(hipEventElapsedTime(elapsed_ms, c->ev_ph0[phase], c->ev_ph1[phase]));
        else *elapsed_ms = -1.f;  // the phase last ran inside a mixed or fused step, which brackets no phase of its own
    }
    return NEXUS_OK;
}

static int mixed_step_impl(nexus_ctx *c, int lb, int le, int handover, const nexus_prefill_batch *pb, const nexus_decode_batch *db,
                           const nexus_kv_cache *kv, void *caller_stream, nexus_step_timing *timing) {
    NX_TRY(check_layers(c, lb, le));
    NX_TRY(check_kv(c, kv, le));
    NX_TRY(check_prefill(c, pb));
    NX_TRY(check_decode(c, db));
    DeviceGuard dg(c->device);
    NX_TRY(debug_validate(c, pb, db, kv));
    Layout *L = c->cur;
    hipStream_t cs = (hipStream_t)caller_stream;
    const bool split = L->sd != L->sp;
    const bool auto_handover = handover == NEXUS_HANDOVER_AUTO;
    nexus_ctx::HandoverSample *sample = nullptr;
    if (auto_handover) {
        handover = le;
        if (split) {
            // phase times of earlier steps that have completed by now
            for (int i = 0; i < 2; ++i) {  // the older set first: the newest completed step has the last word
                auto &hs = c->ho_sample[c->ho_next ^ i];
                if (!hs.pending || hipEventQuery(hs.d1) != hipSuccess || hipEventQuery(hs.ph) != hipSuccess) continue;
                float t_dec = 0.f, t_head = 0.f;
                hs.pending = false;
                if (hipEventElapsedTime(&t_dec, hs.d0, hs.d1) != hipSuccess || hipEventElapsedTime(&t_head, hs.p0, hs.ph) != hipSuccess) continue;
                if (hs.head_layers > 0 && t_head > 0.f && t_dec > 0.f)
                    c->ho_layout = hs.layout, c->ho_decode_ms = t_dec, c->ho_head_layer_ms = t_head / hs.head_layers;
            }
            // the first layer boundary after the decode step's end; without a measurement on this layout the split is
            // held to the end of the step, which produces one
            if (c->ho_layout == L && c->ho_head_layer_ms > 0.f)
                handover = std::max(lb + 1, std::min(le, lb + (int)std::ceil(c->ho_decode_ms / c->ho_head_layer_ms)));
            sample = &c->ho_sample[c->ho_next];
            c->ho_next ^= 1;
        }
    }
    c->last_handover_layer = split ? handover : le;
    if (cs) {
        HIP_TRY(hipEventRecord(c->ev_caller, cs));
        HIP_TRY(hipStreamWaitEvent(L->sp, c->ev_caller, 0));
        if (split) HIP_TRY(hipStreamWaitEvent(L->sd, c->ev_caller, 0));
    }
    // Steps of one context never overlap: both phases of this step follow the previous launch of either phase,
    // whatever layout that ran on (no-ops before the first step and for work on this very stream).  A request that
    // finished prefilling in step n can therefore decode in step n + 1, and a change of layout between two steps
    // needs no synchronisation.
    NX_TRY(order_after(c, L->sp, NEXUS_PHASE_PREFILL));
    NX_TRY(order_after(c, L->sp, NEXUS_PHASE_DECODE));
    if (split) {
        // fork: the decode stream starts when the prefill stream reaches this point, i.e. after everything the
        // prefill stream has just been made to wait for
        HIP_TRY(hipEventRecord(c->ev_fork, L->sp));
        HIP_TRY(hipStreamWaitEvent(L->sd, c->ev_fork, 0));
    }
    if (timing) {
        HIP_TRY(hipEventRecord(c->ev_sp0, L->sp));
        if (split) HIP_TRY(hipEventRecord(c->ev_sd0, L->sd));
    }
    if (sample) {
        HIP_TRY(hipEventRecord(sample->p0, L->sp));
        HIP_TRY(hipEventRecord(sample->d0, L->sd));
        sample->layout = L, sample->head_layers = handover - lb, sample->pending = false;
    }
    const PhaseRun rp = make_run(c, NEXUS_PHASE_PREFILL, pb, nullptr, kv), rd = make_run(c, NEXUS_PHASE_DECODE, nullptr, db, kv);
    if (split) {
        // the two phases are enqueued alternately, a layer of each at a time, the decode phase (whose kernels are the
        // shorter ones) first: both streams have work from the start of the step
        PhaseRun rt = rp;
        if (handover < le) {
            Layout *all = nullptr;
            NX_TRY(get_layout(c, NEXUS_CUS_ALL, NEXUS_CUS_ALL, &all));
            rt.s = all->sp, rt.n_xcd = all->p_xcd, rt.cus = c->n_cus;
        }
        PhaseCursor pc(rp, lb, le, handover < le ? &rt : nullptr, handover), dc(rd, lb, le);
        while (!pc.done() || !dc.done()) {
            if (!dc.done()) {
                NX_TRY(dc.step());
                if (dc.done()) {
                    if (sample) HIP_TRY(hipEventRecord(sample->d1, L->sd));
                    NX_TRY(mark_done(c, L->sd, NEXUS_PHASE_DECODE, false));
                }
            }
            if (!pc.done()) {
                NX_TRY(pc.step());
                if (sample && pc.l == handover) HIP_TRY(hipEventRecord(sample->ph, L->sp));  // end of the layers run on the share
                if (pc.done()) NX_TRY(mark_done(c, pc.last_stream(), NEXUS_PHASE_PREFILL, false));
            }
        }
        if (sample) sample->pending = true;  // all four events of the sample are recorded
    } else {
        NX_TRY(run_phase(rp, lb, le));
        NX_TRY(mark_done(c, L->sp, NEXUS_PHASE_PREFILL, false));
        NX_TRY(run_phase(rd, lb, le));
        NX_TRY(mark_done(c, L->sd, NEXUS_PHASE_DECODE, false));
    }
    if (cs) {
        if (split) HIP_TRY(hipStreamWaitEvent(cs, c->ev_ph1[NEXUS_PHASE_PREFILL], 0));
        HIP_TRY(hipStreamWaitEvent(cs, c->ev_ph1[NEXUS_PHASE_DECODE], 0));
    }
    hipEvent_t ev_sp1 = c->ev_ph1[NEXUS_PHASE_PREFILL], ev_sd1 = c->ev_ph1[NEXUS_PHASE_DECODE];
    if (timing) {
        HIP_TRY(hipEventSynchronize(ev_sp1));
        HIP_TRY(hipEventSynchronize(ev_sd1));
        float tp = 0, td = 0;
        HIP_TRY(hipEventElapsedTime(&tp, c->ev_sp0, ev_sp1));
        if (split) {
            float d0 = 0, pd = 0;
            HIP_TRY(hipEventElapsedTime(&td, c->ev_sd0, ev_sd1));
            HIP_TRY(hipEventElapsedTime(&pd, c->ev_sp0, ev_sd1));  // prefill start -> decode end
            HIP_TRY(hipEventElapsedTime(&d0, c->ev_sp0, c->ev_sd0));  // start skew (may be negative)
            const float start = std::min(0.f, d0);
            timing->t_prefill_ms = tp, timing->t_decode_ms = td;
            timing->t_step_ms = std::max(tp, pd) - start;
        } else {
            HIP_TRY(hipEventElapsedTime(&td, c->ev_sp0, ev_sd1));  // decode waits for prefill: its latency includes it
            timing->t_prefill_ms = tp, timing->t_decode_ms = td, timing->t_step_ms = td;
        }
    }
    return NEXUS_OK;
}

int nexus_mixed_step(nexus_ctx *c, int lb, int le, const nexus_prefill_batch *pb, const nexus_decode_batch *db, const nexus_kv_cache *kv,
                     void *caller_stream, nexus_step_timing *timing) {
    return mixed_step_impl(c, lb, le, le, pb, db, kv, caller_stream, timing);
}

int nexus_mixed_step_handover(nexus_ctx *c, int lb, int le, int handover_layer, const nexus_prefill_batch *pb, const nexus_decode_batch *db,
                              const nexus_kv_cache *kv, void *caller_stream, nexus_step_timing *timing) {
    if (handover_layer != NEXUS_HANDOVER_AUTO && (handover_layer < lb || handover_layer > le))
        return fail(NEXUS_EINVAL, "handover layer %d outside [%d, %d]", handover_layer, lb, le);
    return mixed_step_impl(c, lb, le, handover_layer, pb, db, kv, caller_stream, timing);
}

int nexus_last_handover_layer(nexus_ctx *c) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    return c->last_handover_layer;
}

static float median(std::vector<float> v) {
    std::sort(v.begin(), v.end());
    return v[v.size() / 2];
}

static int time_phase(nexus_ctx *c, int phase, int lb, int le, const nexus_prefill_batch *pb, const nexus_decode_batch *db, const nexus_kv_cache *kv,
                      int repeats, float *out_ms) {
    std::vector<float> t;
    hipStream_t s = phase == NEXUS_PHASE_PREFILL ? c->cur->sp : c->cur->sd;
    for (int i = 0; i < repeats + 1; ++i) {
        HIP_TRY(hipEventRecord(c->ev_sp0, s));
        NX_TRY(run_phase(make_run(c, phase, pb, db, kv), lb, le));
        HIP_TRY(hipEventRecord(c->ev_sp1, s));
        HIP_TRY(hipStreamSynchronize(s));
        float ms = 0;
        HIP_TRY(hipEventElapsedTime(&ms, c->ev_sp0, c->ev_sp1));
        if (i) t.push_back(ms);  // first run is the warm-up
    }
    *out_ms = median(t);
    return NEXUS_OK;
}

int nexus_profile_split(nexus_ctx *c, int lb, int le, const nexus_prefill_batch *pb, const nexus_decode_batch *db, const nexus_kv_cache *kv,
                        const int32_t *cand, int n_cand, int policy, float alpha, float beta, int repeats, float *t_p, float *t_d, float *t_s,
                        float *t_all, int32_t *chosen) {
    NX_TRY(check_layers(c, lb, le));
    NX_TRY(check_kv(c, kv, le));
    NX_TRY(check_prefill(c, pb));
    NX_TRY(check_decode(c, db));
    if (!cand || n_cand <= 0 || !t_p || !t_d || !t_s || !t_all || !chosen) return fail(NEXUS_EINVAL, "null output or no candidates");
    if (policy < 0 || policy > 2) return fail(NEXUS_EINVAL, "unknown policy %d", policy);
    if (repeats <= 0) return fail(NEXUS_EINVAL, "repeats must be positive");
    const int gran = c->n_xcd;
    for (int i = 0; i < n_cand; ++i)
        if (cand[i] <= 0 || cand[i] >= c->n_cus || cand[i] % gran || (c->n_cus - cand[i]) % gran)
            return fail(NEXUS_EINVAL, "candidate %d (%d prefill CUs) is not a valid split of %d CUs at granularity %d", i, cand[i], c->n_cus, gran);
    DeviceGuard dg(c->device);
    NX_TRY(nexus_sync(c));
    NX_TRY(nexus_set_cu_split(c, NEXUS_CUS_ALL, NEXUS_CUS_ALL));
    NX_TRY(time_phase(c, NEXUS_PHASE_PREFILL, lb, le, pb, nullptr, kv, repeats, &t_all[0]));
    NX_TRY(time_phase(c, NEXUS_PHASE_DECODE, lb, le, nullptr, db, kv, repeats, &t_all[1]));
    for (int i = 0; i < n_cand; ++i) {
        NX_TRY(nexus_set_cu_split(c, cand[i], c->n_cus - cand[i]));
        NX_TRY(time_phase(c, NEXUS_PHASE_PREFILL, lb, le, pb, nullptr, kv, repeats, &t_p[i]));
        NX_TRY(time_phase(c, NEXUS_PHASE_DECODE, lb, le, nullptr, db, kv, repeats, &t_d[i]));
        std::vector<float> ts;
        for (int k = 0; k < repeats + 1; ++k) {
            nexus_step_timing tm;
            NX_TRY(nexus_mixed_step(c, lb, le, pb, db, kv, nullptr, &tm));
            if (k) ts.push_back(tm.t_step_ms);
        }
        t_s[i] = median(ts);
    }
    const int best = nexus_choose_split(n_cand, t_p, t_d, t_s, t_all[0], t_all[1], policy, alpha, beta);
    if (best < 0) return best;
    *chosen = cand[best];
    return nexus_set_cu_split(c, cand[best], c->n_cus - cand[best]);
}

int nexus_trace_begin(nexus_ctx *c, int phase, int kernel) {
    if (!c) return fail(NEXUS_EINVAL, "null context");
    if (phase < 0 || phase > 1 || kernel < 0 || kernel >= NEXUS_K_COUNT) return fail(NEXUS_EINVAL, "bad phase / kernel id");
    DeviceGuard dg(c->device);
    if (c->trace_pool.empty()) {
        c->trace_pool.resize(4096);
        for (auto &t : c->trace_pool) {
            HIP_TRY(hipEventCreateWithFlags(&t.a, hipEventDisableSystemFence));
            HIP_TRY(hipEventCreateWithFlags(&t.b, hipEventDisableSystemFence));
        }
    }
    c->trace_used = 0;
    c->trace_phase = phase, c->trace_kernel = kernel;
    return NEXUS_OK;
}

int nexus_trace_read(nexus_ctx *c, float *mean_ms, int32_t *launches) {
    if (!c || !mean_ms || !launches) return fail(NEXUS_EINVAL, "null argument");
    DeviceGuard dg(c->device);
    c->trace_phase = c->trace_kernel = -1;
    NX_TRY(nexus_sync(c));
    double sum = 0;
    for (size_t i = 0; i < c->trace_used; ++i) {
        float ms = 0;
        HIP_TRY(hipEventElapsedTime(&ms, c->trace_pool[i].a, c->trace_pool[i].b));
        sum += ms;
    }
    *launches = (int32_t)c->trace_used;
    *mean_ms = c->trace_used ? (float)(sum / c->trace_used) : 0.f;
    c->trace_used = 0;
    return NEXUS_OK;
}

int nexus_debug_fetch(nexus_ctx *c, int phase, int which, int32_t n_tokens, void *out) {
    if (!c || !out) return fail(NEXUS_EINVAL, "null argument");
    if (phase < 0 || phase > 1) return fail(NEXUS_EINVAL, "bad phase");
    PhaseWs &w = c->ws[phase];
    if (n_tokens <= 0 || n_tokens > w.maxT) return fail(NEXUS_EINVAL, "n_tokens outside the workspace");
    DeviceGuard dg(c->device);
    NX_TRY(nexus_sync(c));
    const void *src = nullptr;
    int K = 0, kind = 0;  // 0 half P32, 1 bf16 P32, 2 half row-major, 3 bf16 row-major
    switch (which) {
        case NEXUS_BUF_NORM1: return fail(NEXUS_ESTATE, "the first norm's output is overwritten by the second norm within a layer");
        case NEXUS_BUF_Q: src = w.q, K = c->q_dim, kind = phase == NEXUS_PHASE_PREFILL ? 1 : 3; break;
        case NEXUS_BUF_ATTN: src = w.attn, K = c->q_dim, kind = 0; break;
        case NEXUS_BUF_X1: src = w.x1, K = c->m.hidden, kind = -1; break;
        case NEXUS_BUF_ACT: src = w.act, K = c->m.ffn, kind = 0; break;
        default: return fail(NEXUS_EINVAL, "unknown buffer id %d", which);
    }
    if (kind < 0) {
        HIP_TRY(hipMemcpyAsync(out, src, (size_t)n_tokens * K * 4, hipMemcpyDeviceToDevice, c->s_main));
    } else {
        // prefill queries sit in request-aligned tiles; callers with one request (or 32-aligned chunks) see rows in order
        const size_t n = (size_t)n_tokens * K;
        hipLaunchKernelGGL(debug_to_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->s_main, (const unsigned short *)src, (float *)out,
                           n_tokens, K, p32_kp(K), kind);
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipStreamSynchronize(c->s_main));
    return NEXUS_OK;
}

int nexus_debug_cu_probe(nexus_ctx *c, int phase, int n_blocks, int32_t *out_counts) {
    if (!c || !out_counts) return fail(NEXUS_EINVAL, "null argument");
    if (phase < 0 || phase > 1 || n_blocks <= 0 || n_blocks > (1 << 20)) return fail(NEXUS_EINVAL, "bad phase or block count");
    DeviceGuard dg(c->device);
    hipStream_t s = phase == NEXUS_PHASE_PREFILL ? c->cur->sp : c->cur->sd;
    HIP_TRY(hipMemsetAsync(c->probe_counts, 0, 8 * 128 * sizeof(int32_t), s));
    hipLaunchKernelGGL(cu_probe_kernel, dim3(n_blocks), dim3(64), 0, s, c->probe_counts);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipMemcpy(out_counts, c->probe_counts, 8 * 128 * sizeof(int32_t), hipMemcpyDeviceToHost));
    return NEXUS_OK;
}

}  // extern "C"
