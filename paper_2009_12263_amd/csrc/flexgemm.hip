// C ABI of libflexgemm.so: argument validation, the "params" choice (Section 4.2.1: which block
// tile and kernel variant serve a problem) and the launch.  All arithmetic of the method runs in
// the kernels of gemm_kernel.hpp; this file only describes problems to them.
#include "../../include/flexgemm.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "kernel_table.hpp"

namespace {

thread_local char g_err[512] = "";

fg_status fail(fg_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned_to(const void *p, unsigned bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; }

// Requirements of the tiled kernels that the general kernel does not have (16-byte aligned bases,
// leading dimensions in whole 16-byte chunks, K a multiple of 8).  A call that misses one of them
// is noted here while it is validated; plain real products then run on the general kernel, every
// other kind of product fails with the noted status and message.
struct Relaxed { fg_status status; char msg[256]; };
thread_local Relaxed g_relaxed = {FG_OK, ""};

void note_relaxed(fg_status st, const char *fmt, ...) {
    if (g_relaxed.status != FG_OK) return;          // keep the first
    g_relaxed.status = st;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_relaxed.msg, sizeof g_relaxed.msg, fmt, ap);
    va_end(ap);
}

constexpr int kNumCU = 256;   // MI355X: 8 XCDs x 32 compute units

// Tuning overrides of the planner, from the environment: FG_FORCE_TILE=0..5 picks a tile shape (0..2
// for the three tiles of the complex and dual kernels)
// (5: the 256x256 tile with the k32 kernel where the family has one), FG_FORCE_SPLIT=n a split of K
// for every tile, FG_FORCE_TAIL=n a split of K for the tiles of the last round (1: never).  Read
// when the library is loaded and again by fg_reload_tuning(), not on every call.
std::atomic<int> g_force_tile{-1}, g_force_split{0}, g_force_tail{0};

void read_tuning_from_environment() {
    const char *t = getenv("FG_FORCE_TILE"), *s = getenv("FG_FORCE_SPLIT"), *l = getenv("FG_FORCE_TAIL");
    g_force_tile.store(t ? atoi(t) : -1);
    g_force_split.store(s ? atoi(s) : 0);
    g_force_tail.store(l ? atoi(l) : 0);
}
struct TuningAtLoad { TuningAtLoad() { read_tuning_from_environment(); } } g_tuning_at_load;

// ---- description of one GEMM after normalisation to "column-major D" ------------------------
struct Problem {
    int64_t M, N, K;
    const void *A, *A_im, *B, *B_im;
    bool a_kc, b_kc;         // operand is K-contiguous
    bool a_diag, b_diag;
    int64_t lda, ldb;
    const float *C, *C_im;
    float *D, *D_im;
    int64_t ldc, ldd;
    const float *bias;
    int bias_dim, act;
    float alpha, beta;
    bool cplx;               // two planes per operand: complex, or dual when `dual` is set
    bool dual;
    bool bf16;               // A and B hold bfloat16
    int c_act;               // activation on loaded C
    uint16_t a_add, b_add;   // FP16 bit patterns of the addends on loaded A and B; ab_add: in use
    bool ab_add;
    bool ilv;                // complex matrices in interleaved storage
    bool general;            // operands miss a requirement of the tiled kernels: use the general kernel
    bool cd16;               // C and D hold binary16 (converted when loaded / stored)
};

// What to launch for a normalised problem: block tile, and into how many K ranges the product is
// split (1: one pass; more: partial products into the workspace, then the reduction pass).
// tail_splits > 1: the tiles that fill whole rounds of the persistent grid are computed in one
// pass, and only the tiles of the last, partly filled round are split over K.
struct Plan { int tile; int splits; int tail_splits; };

constexpr int64_t kWorkspaceBytes = 64ll << 20;    // split-K partial products, per device

const fg::KernelEntry *table_h16_for(bool a_kc, bool b_kc) {
    if (!a_kc && b_kc) return fg::kernel_table_nn_h16();
    if (!a_kc && !b_kc) return fg::kernel_table_nt_h16();
    if (a_kc && b_kc) return fg::kernel_table_tn_h16();
    return fg::kernel_table_tt_h16();
}

const fg::KernelEntry *table_for(bool a_kc, bool b_kc) {
    if (!a_kc && b_kc) return fg::kernel_table_nn();
    if (!a_kc && !b_kc) return fg::kernel_table_nt();
    if (a_kc && b_kc) return fg::kernel_table_tn();
    return fg::kernel_table_tt();
}

// The params heuristic (Section 4.2.1 picks the largest tile that fits shared memory; here every
// tile fits, so the question is which shape, and which split of K, finishes first).  Estimated
// time = rounds x (time of one workgroup on its share of K + the time of its epilogue) + the cost
// of the reduction pass if K is split.  `rounds` = ceil(workgroups / slots), slots = 256 compute
// units x workgroups of that shape per unit; a workgroup's rate is a measured fraction of what a
// compute unit sustains with the 256x256 tile (about 4.7 TFLOP/s), one set for workgroups that
// share a unit and one for a workgroup that has a unit to itself.  Edge tiles are predicated, so
// a tile need not divide the problem.  K is split only when the output has too few tiles to fill
// the GPU and K is long (may_split: plain real products).
// k32: the kernel family has the 256x256 tile with 16x16x32 matrix instructions
// (TILE_256x256_K32).  It is not a candidate of its own.  k32 == 2: it replaces the 256x256 tile
// when that one is chosen and the output has such a tile for at least three quarters of the
// compute units (measured +1 to +5 % from 192 tiles up, K from 1024 to 8192; equal at 176 tiles,
// -1 to -6 % at 160 and fewer: a partly busy chip is not at its power limit).  k32 == 1: only
// when forced (A and B both M/N-contiguous: measured 0 to -5 %).
Plan choose_plan(int64_t M, int64_t N, int64_t K, bool may_split, bool allow_smallest = true, int64_t batches = 1,
                 bool allow_deep = true, int k32 = 0) {
    static const int bm[fg::TILE_COUNT] = {256, 256, 128, 64, 128, 256};
    static const int bn[fg::TILE_COUNT] = {256, 128, 128, 64, 128, 256};
    static const int per_cu[fg::TILE_COUNT] = {1, 1, 2, 4, 1, 1};
    static const double rate_shared[fg::TILE_COUNT] = {1.0, 0.8, 0.73, 0.45, 0.57, 1.0};
    static const double rate_alone[fg::TILE_COUNT] = {1.0, 0.8, 0.43, 0.17, 0.57, 1.0};
    static const int split_options[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64};
    constexpr double cu_flops = 4.7e12, round_fixed = 2e-6, cu_cd_bw = 25e9, reduce_launch = 6e-6, reduce_bw = 3e12;
    // tuning overrides (see read_tuning_from_environment)
    int force_tile = -1;
    const int force_split = g_force_split.load(std::memory_order_relaxed), force_tail = g_force_tail.load(std::memory_order_relaxed);
    bool force_k32 = false, forced_plain = false;
    {
        int t = g_force_tile.load(std::memory_order_relaxed);
        if (t == fg::TILE_256x256_K32) { t = fg::TILE_256x256; force_k32 = true; }
        else forced_plain = (t == fg::TILE_256x256);
        if (t >= 0 && t < fg::TILE_COUNT) force_tile = t;
    }
    const int64_t nk = (K + 63) / 64;                       // K tiles (every real kernel has BK = 64)
    Plan best{0, 1, 1};
    double best_cost = -1;
    for (int t = 0; t < fg::TILE_COUNT; ++t) {
        if (force_tile >= 0 && t != force_tile) continue;
        if (t == fg::TILE_64x64 && !allow_smallest) continue;
        if (t == fg::TILE_128x128_DEEP && !allow_deep) continue;
        if (t == fg::TILE_256x256_K32) continue;
        const int64_t tiles = ((M + bm[t] - 1) / bm[t]) * ((N + bn[t] - 1) / bn[t]) * batches;
        const int64_t slots = (int64_t)kNumCU * per_cu[t];
        const int64_t slot_bytes = (int64_t)bm[t] * bn[t] * 4;
        auto share_time = [&](int64_t wgs, int S) {     // one workgroup on 1/S of K, plus its epilogue
            // workgroups that share a compute unit at a time: a unit's rate grows linearly from the
            // lone-workgroup rate to the rate with every slot taken, and is divided among them
            int64_t n = (wgs + kNumCU - 1) / kNumCU;
            if (n > per_cu[t]) n = per_cu[t];
            const double unit_rate = per_cu[t] == 1 ? rate_alone[t]
                                   : rate_alone[t] + (rate_shared[t] - rate_alone[t]) * (double)(n - 1) / (per_cu[t] - 1);
            const double rate = unit_rate / (double)n;
            // the C read and D write of a tile stream at what one compute unit gets of the memory
            // bandwidth, divided among the workgroups that share the unit
            const double epilogue = round_fixed + (double)n * 8.0 * bm[t] * bn[t] / cu_cd_bw;
            return 2.0 * bm[t] * bn[t] * (double)((nk + S - 1) / S) * 64 / (cu_flops * rate) + epilogue;
        };
        auto reduce_time = [&](int64_t ntile, int S) { return reduce_launch + (2.0 * S + 2.0) * (double)ntile * slot_bytes / reduce_bw; };
        auto consider = [&](int S, int tail, double cost) {
            if (best_cost < 0 || cost < best_cost) { best = Plan{t, S, tail}; best_cost = cost; }
        };
        // (a) every tile split S ways (S = 1: the plain launch)
        auto legal = [&](int S) { return S == 1 || (may_split && S <= nk && tiles * S * slot_bytes <= kWorkspaceBytes); };
        const int forced = (force_split >= 1 && legal(force_split)) ? force_split : (force_split >= 1 ? 1 : 0);
        for (int S : split_options) {
            if (forced) { if (S != split_options[0]) break; S = forced; }      // one candidate: the forced split
            else if (S > 1 && (!legal(S) || nk / S < 4)) break;                   // at least 256 k per share
            const int64_t wgs = tiles * S;
            const int64_t rounds = (wgs + slots - 1) / slots;
            double cost = (double)rounds * share_time(wgs, S);
            if (S > 1) cost += reduce_time(tiles, S);
            consider(S, 1, cost);
        }
        // (b) whole rounds in one pass, the tiles of the last, partly filled round split over K
        const int64_t full = tiles / slots * slots, rest = tiles - full;
        if (may_split && full > 0 && rest > 0 && force_split < 1 && force_tail != 1) {
            for (int S : split_options) {
                if (S == 1) continue;
                if (force_tail > 1) { if (S != split_options[1]) break; S = force_tail; }
                const bool fits = S <= nk && rest * S * slot_bytes <= kWorkspaceBytes;
                if (force_tail > 1) { if (!fits) break; }
                else if (!fits || nk / S < 4 || rest * S > slots) break;
                const double cost = (double)(full / slots) * share_time(full, 1) + 2e-6 +
                                    (double)((rest * S + slots - 1) / slots) * share_time(rest * S, S) + reduce_time(rest, S);
                consider(1, S, force_tail > 1 ? 0.0 : cost);
            }
        }
    }
    // A short K (up to 256) makes the product a pass over C and D: there the 256x128 tile measured
    // 4 to 15 % faster than the 256x256 tile the estimate picks (8192^2 x 64: 95.7 against 100.3 us,
    // 4096^2 x 128: 27.9 against 29.8, 8192^2 x 256: 107.1 against 112.1; at K = 384 and 512 it
    // wins with a C operand and loses without one, from K = 768 on it loses).  Matrix kernels only,
    // which is what k32 > 0 says: contraction 5a, K = 256, is faster on the larger tile.
    if (best.tile == fg::TILE_256x256 && k32 > 0 && force_tile < 0 && nk <= 4 && best.splits == 1 && best.tail_splits == 1)
        best.tile = fg::TILE_256x128;
    if (best.tile == fg::TILE_256x256 && k32 > 0 && !forced_plain) {
        const int64_t tiles = ((M + 255) / 256) * ((N + 255) / 256) * batches;
        if (force_k32 || (k32 == 2 && tiles >= kNumCU * 3 / 4)) best.tile = fg::TILE_256x256_K32;
    }
    return best;
}

// Tile of the complex and dual kernels (256x128, 128x128 with two workgroups per unit, 64x64 with
// four): the one with the smallest estimated time.  Whole rounds run with every slot of a unit
// taken, the workgroups of the last, partly filled round share a unit with fewer others; a
// workgroup's rate is a measured fraction of what a unit sustains with the 256x128 tile (4096^3:
// 455 / 515 / 629 us with the three tiles; alone on a unit: 1024^3 51 / 35 / 18 us).  The estimate
// reproduces the fastest tile of every measured case but one near-tie (2560^3: 131 us against 156 us
// for the tile the former rule, "the largest tile with 256 tiles", picked; 3072^3: 276 against 301).
int choose_ctile(int64_t M, int64_t N) {
    static const int bm[fg::CTILE_COUNT] = {256, 128, 64};
    static const int bn[fg::CTILE_COUNT] = {128, 128, 64};
    static const int per_cu[fg::CTILE_COUNT] = {1, 2, 4};
    static const double rate_shared[fg::CTILE_COUNT] = {1.0, 0.883, 0.72};
    static const double rate_alone[fg::CTILE_COUNT] = {1.0, 0.74, 0.45};
    const int forced = g_force_tile.load(std::memory_order_relaxed);      // tuning override, 0..2 here
    if (forced >= 0 && forced < fg::CTILE_COUNT) return forced;
    int best = 0;
    double best_cost = -1;
    for (int t = 0; t < fg::CTILE_COUNT; ++t) {
        const int64_t tiles = ((M + bm[t] - 1) / bm[t]) * ((N + bn[t] - 1) / bn[t]);
        const int64_t slots = (int64_t)kNumCU * per_cu[t];
        auto tile_time = [&](int64_t sharing) {     // one tile, `sharing` workgroups on its unit
            const double unit = per_cu[t] == 1 ? rate_alone[t]
                              : rate_alone[t] + (rate_shared[t] - rate_alone[t]) * (double)(sharing - 1) / (per_cu[t] - 1);
            return (double)bm[t] * bn[t] * (double)sharing / unit;
        };
        const int64_t full = tiles / slots, rest = tiles - full * slots;
        double cost = (double)full * tile_time(per_cu[t]);
        if (rest > 0) cost += tile_time((rest + kNumCU - 1) / kNumCU);
        if (best_cost < 0 || cost < best_cost) { best = t; best_cost = cost; }
    }
    return best;
}

// Kernel variant for a normalised problem.
const fg::KernelEntry *select_kernel(const Problem &q, Plan *plan_out = nullptr) {
    if (plan_out) *plan_out = Plan{0, 1, 1};
    if (q.cplx) {
        const int t = choose_ctile(q.M, q.N);
        if (t < 0) return nullptr;
        const int v = (q.a_kc ? 2 : 0) + (q.b_kc ? 0 : 1);     // nn, nt, tn, tt
        if (q.ilv) return &fg::kernel_table_cplx_il()[t * 4 + v];
        return &(q.dual ? fg::kernel_table_dual() : fg::kernel_table_cplx())[t * 4 + v];
    }
    const bool may_split = plan_out && !q.a_diag && !q.b_diag && !q.cd16;   // the reduction pass writes FP32
    const int k32 = (q.a_diag || q.b_diag) ? 0 : q.ab_add ? (q.a_kc != q.b_kc ? 2 : 0) : ((q.a_kc || q.b_kc) ? 2 : 1);
    const Plan plan = choose_plan(q.M, q.N, q.K, may_split, true, 1, !q.a_diag && !q.b_diag, k32);
    int tile = plan.tile;
    // A product with a diagonal operand is bound by its memory traffic (one pass over the dense
    // operand, C and D; a tile row only meets the K tiles on the diagonal).  While all of it fits the
    // 256 MB memory-side cache, the smallest tile, four workgroups per unit at different points
    // between their loads and their stores, measured fastest (4096^2: 26.6 us against 29.6 us with
    // the 256x256 tile, 8192 x 1024: 14.8 against 17.0); beyond that size its short pieces cost
    // more in memory than they gain (8192^2: 180 us against 135 us), and the estimate above decides.
    if ((q.a_diag || q.b_diag) && g_force_tile.load(std::memory_order_relaxed) < 0 && q.M * q.N * 10 <= (256ll << 20))
        tile = fg::TILE_64x64;
    if (plan_out) { *plan_out = plan; plan_out->tile = tile; }
    if (q.a_diag) return &fg::kernel_table_diag()[tile * 4 + (q.b_kc ? 0 : 1)];
    if (q.b_diag) return &fg::kernel_table_diag()[tile * 4 + (q.a_kc ? 2 : 3)];
    if (q.ab_add) {
        const fg::KernelEntry *t = !q.a_kc ? (q.b_kc ? fg::kernel_table_nn_xf() : fg::kernel_table_nt_xf())
                                           : (q.b_kc ? fg::kernel_table_tn_xf() : fg::kernel_table_tt_xf());
        return &t[tile];
    }
    if (q.cd16) return &table_h16_for(q.a_kc, q.b_kc)[tile];
    if (q.bf16) {
        const fg::KernelEntry *t = !q.a_kc ? (q.b_kc ? fg::kernel_table_nn_bf16() : fg::kernel_table_nt_bf16())
                                           : (q.b_kc ? fg::kernel_table_tn_bf16() : fg::kernel_table_tt_bf16());
        return &t[tile];
    }
    return &table_for(q.a_kc, q.b_kc)[fg::entry_index(tile, fg::VARIANT_MATRIX)];
}

// Once per (kernel, device): raise the dynamic LDS limit and ask how many workgroups of this
// kernel fit on a compute unit.
fg_status prepare(const fg::KernelEntry &k, int dev, int &per_cu) {
    static std::mutex m;
    static struct { const void *fn; int dev; int per_cu; } done[512];
    static int n_done = 0;
    std::lock_guard<std::mutex> lock(m);
    per_cu = 0;
    for (int i = 0; i < n_done; ++i)
        if (done[i].fn == (const void *)k.fn && done[i].dev == dev) per_cu = done[i].per_cu;
    if (per_cu == 0) {
        hipError_t e = hipFuncSetAttribute((const void *)k.fn, hipFuncAttributeMaxDynamicSharedMemorySize, k.lds_bytes);
        if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "hipFuncSetAttribute(%s): %s", k.name, hipGetErrorString(e));
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)k.fn, k.threads, (size_t)k.lds_bytes);
        if (e != hipSuccess || per_cu < 1) return fail(FG_ERR_LAUNCH, "occupancy query for %s failed: %s", k.name, hipGetErrorString(e));
        if (n_done < 512) { done[n_done].fn = (const void *)k.fn; done[n_done].dev = dev; done[n_done].per_cu = per_cu; ++n_done; }
    }
    return FG_OK;
}

// Split-K workspace: one allocation of kWorkspaceBytes per device, made by fg_init() or by the
// first call that splits K, and kept until the process ends.  Every split-K call on a device
// uses it.  Calls on one stream are ordered anyway; a call on another stream than the previous
// user's first waits (on the device, not on the host) for the event that user recorded after its
// reduction pass, so that calls on different streams cannot overwrite each other's partial
// products.  A stream that is being captured into a graph takes no part in this (events recorded
// into a graph order nothing outside it): captured split-K calls must be ordered by the caller,
// and the workspace must exist before the capture starts (fg_init()).
struct Workspace {
    float *ptr = nullptr;
    hipEvent_t last_use = nullptr;       // recorded after the most recent split-K call's reduction pass
    hipStream_t last_stream = nullptr;
    bool used = false;
};
std::mutex g_ws_mutex;
Workspace g_ws[64];

bool stream_is_capturing(hipStream_t stream) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
    return st != hipStreamCaptureStatusNone;
}

// Must be called with g_ws_mutex held.
fg_status workspace_locked(int dev, hipStream_t stream, bool may_allocate, Workspace **out) {
    if (dev < 0 || dev >= 64) return fail(FG_ERR_LAUNCH, "device index %d out of range", dev);
    Workspace &w = g_ws[dev];
    if (!w.ptr) {
        if (!may_allocate || stream_is_capturing(stream))
            return fail(FG_ERR_UNSUPPORTED, "this call splits K and needs the library's workspace, which cannot be allocated while the "
                                            "stream is being captured: call fg_init() on this device before the capture");
        void *ptr = nullptr;
        hipError_t e = hipMalloc(&ptr, (size_t)kWorkspaceBytes);
        if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "hipMalloc of the split-K workspace failed: %s", hipGetErrorString(e));
        e = hipEventCreateWithFlags(&w.last_use, hipEventDisableTiming);
        if (e != hipSuccess) { (void)hipFree(ptr); return fail(FG_ERR_LAUNCH, "hipEventCreate for the split-K workspace failed: %s", hipGetErrorString(e)); }
        w.ptr = (float *)ptr;
    }
    *out = &w;
    return FG_OK;
}

// The allocation-free entry point keeps its partial products in this array instead: part of the
// library's device image, so each GPU the library runs on holds one copy until the process ends.
// Host code never uses the symbol itself as an address: g_static_scratch[dev] is the array's
// device address on GPU `dev`, asked for once per device with that device current.
constexpr int64_t kStaticScratchBytes = 16ll << 20;
static __device__ __align__(256) float scratch[kStaticScratchBytes / 4];
float *g_static_scratch[64];

fg_status static_scratch(int dev, float **out) {
    static std::mutex m;
    if (dev < 0 || dev >= 64) return fail(FG_ERR_LAUNCH, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(m);
    if (!g_static_scratch[dev]) {
        float *ptr = nullptr;
        hipError_t e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail(FG_ERR_LAUNCH, "hipGetSymbolAddress of the static scratch array failed: %s", hipGetErrorString(e));
        g_static_scratch[dev] = ptr;
    }
    *out = g_static_scratch[dev];
    return FG_OK;
}

fg_status launch(const fg::KernelEntry &k, const fg::GemmParams &p, hipStream_t stream) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FG_ERR_LAUNCH, "no HIP device is current");
    int per_cu = 0;
    if (fg_status st = prepare(k, dev, per_cu)) return st;
    // Persistent workgroups: as many as the GPU holds at once; each walks tiles b, b + grid, ...
    const int ntiles = p.tile_count > 0 ? p.tile_count * (p.splits > 1 ? p.splits : 1)
                                        : p.tiles_m * p.tiles_n * (p.batches > 1 ? p.batches : 1);
    const int resident = per_cu * kNumCU;
    dim3 grid((unsigned)(ntiles < resident ? ntiles : resident)), block((unsigned)k.threads);
    hipLaunchKernelGGL(k.fn, grid, block, (size_t)k.lds_bytes, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "launch of %s failed: %s", k.name, hipGetErrorString(e));
    return FG_OK;
}

fg_status check_sizes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return fail(FG_ERR_SHAPE, "negative size M=%lld N=%lld K=%lld", (long long)M, (long long)N, (long long)K);
    if (K % 8) note_relaxed(FG_ERR_UNSUPPORTED, "K must be a multiple of 8 (got %lld)", (long long)K);
    if (M > (1 << 30) || N > (1 << 30) || K > (1 << 30)) return fail(FG_ERR_UNSUPPORTED, "sizes above 2^30 are not supported");
    return FG_OK;
}

fg_status check_input_matrix(const char *name, const fg_matrix *X, int64_t rows, int64_t cols) {
    if (!X) return fail(FG_ERR_NULL, "%s is NULL", name);
    if (X->dtype != FG_F16 && X->dtype != FG_BF16 && X->dtype != FG_CF16) return fail(FG_ERR_LAYOUT, "%s must be FG_F16, FG_BF16 or FG_CF16", name);
    if (X->dtype == FG_CF16 && (X->im || X->layout == FG_DIAG)) return fail(FG_ERR_LAYOUT, "%s: an interleaved complex matrix has no `im` plane and is not diagonal", name);
    if (X->layout != FG_COL && X->layout != FG_ROW && X->layout != FG_DIAG) return fail(FG_ERR_LAYOUT, "%s: layout %d is not valid for an input", name, X->layout);
    if (rows > 0 && cols > 0) {
        if (!X->re) return fail(FG_ERR_NULL, "%s->re is NULL", name);
        if (!aligned_to(X->re, 2) || (X->im && !aligned_to(X->im, 2))) return fail(FG_ERR_ALIGN, "%s: element pointers must be aligned to an element", name);
        if (!aligned16(X->re) || (X->im && !aligned16(X->im))) note_relaxed(FG_ERR_ALIGN, "%s: element pointers must be 16-byte aligned", name);
        if (X->layout != FG_DIAG) {
            int64_t need = X->layout == FG_COL ? rows : cols;
            if (X->ld < need) return fail(FG_ERR_SHAPE, "%s: ld=%lld is smaller than %lld", name, (long long)X->ld, (long long)need);
            if (X->ld % 8) note_relaxed(FG_ERR_ALIGN, "%s: ld=%lld must be a multiple of 8", name, (long long)X->ld);
        }
    }
    return FG_OK;
}

fg_status check_output_matrix(const char *name, const fg_matrix *X, int64_t rows, int64_t cols, bool need_im) {
    if (X->dtype != FG_F32 && X->dtype != FG_CF32 && X->dtype != FG_F16) return fail(FG_ERR_LAYOUT, "%s must be FG_F32, FG_F16 or FG_CF32", name);
    if (X->dtype == FG_F16) {
        // stored as binary16: the kernels access it element by element, so any ld and any
        // element-aligned pointer will do
        if (X->im) return fail(FG_ERR_UNSUPPORTED, "%s: binary16 storage is for real matrices", name);
        if (X->layout != FG_COL && X->layout != FG_ROW) return fail(FG_ERR_LAYOUT, "%s: layout %d is not valid here", name, X->layout);
        if (rows > 0 && cols > 0) {
            if (!X->re) return fail(FG_ERR_NULL, "%s->re is NULL", name);
            if (!aligned_to(X->re, 2)) return fail(FG_ERR_ALIGN, "%s: element pointers must be aligned to an element", name);
            const int64_t need = X->layout == FG_COL ? rows : cols;
            if (X->ld < need) return fail(FG_ERR_SHAPE, "%s: ld=%lld is smaller than %lld", name, (long long)X->ld, (long long)need);
        }
        return FG_OK;
    }
    if (X->dtype == FG_CF32) {
        if (X->im) return fail(FG_ERR_LAYOUT, "%s: an interleaved complex matrix has no `im` plane", name);
        need_im = false;
        if (X->ld >= (1ll << 22)) return fail(FG_ERR_UNSUPPORTED, "%s: ld of an interleaved complex matrix must be below 2^22", name);
    }
    if (X->layout != FG_COL && X->layout != FG_ROW) return fail(FG_ERR_LAYOUT, "%s: layout %d is not valid here", name, X->layout);
    if (rows > 0 && cols > 0) {
        if (!X->re) return fail(FG_ERR_NULL, "%s->re is NULL", name);
        if (need_im && !X->im) return fail(FG_ERR_NULL, "%s->im is NULL but the product is complex", name);
        if (!aligned_to(X->re, 4) || (X->im && !aligned_to(X->im, 4))) return fail(FG_ERR_ALIGN, "%s: element pointers must be aligned to an element", name);
        if (!aligned16(X->re) || (X->im && !aligned16(X->im))) note_relaxed(FG_ERR_ALIGN, "%s: element pointers must be 16-byte aligned", name);
        int64_t need = X->layout == FG_COL ? rows : cols;
        if (X->ld < need) return fail(FG_ERR_SHAPE, "%s: ld=%lld is smaller than %lld", name, (long long)X->ld, (long long)need);
        if (X->ld % 4) note_relaxed(FG_ERR_ALIGN, "%s: ld=%lld must be a multiple of 4", name, (long long)X->ld);
    }
    return FG_OK;
}

// Validate an fg_gemm call and normalise it so that D is column-major: a row-major D is the
// column-major D^T = op(B)^T op(A)^T, i.e. the same kernel with the operands exchanged.
fg_status normalise(int64_t M, int64_t N, int64_t K, float alpha, const fg_matrix *A, const fg_matrix *B,
                    float beta, const fg_matrix *C, const fg_matrix *D, const fg_epilogue *ep, bool dual,
                    const fg_load_transforms *lt, Problem &q) {
    g_relaxed.status = FG_OK;
    if (fg_status st = check_sizes(M, N, K)) return st;
    if (fg_status st = check_input_matrix("A", A, M, K)) return st;
    if (fg_status st = check_input_matrix("B", B, K, N)) return st;
    if (!D) return fail(FG_ERR_NULL, "D is NULL");
    if (A->dtype != B->dtype) return fail(FG_ERR_UNSUPPORTED, "A and B must have the same element type");
    const bool bf16 = A->dtype == FG_BF16;
    const bool ilv = A->dtype == FG_CF16;
    if (ilv && (D->dtype != FG_CF32 || (C && C->layout != FG_ZERO && C->re && C->dtype != FG_CF32)))
        return fail(FG_ERR_UNSUPPORTED, "interleaved complex A and B need interleaved complex (FG_CF32) C and D");
    if (!ilv && (D->dtype == FG_CF32 || (C && C->dtype == FG_CF32 && C->layout != FG_ZERO && C->re)))
        return fail(FG_ERR_UNSUPPORTED, "FG_CF32 C and D need FG_CF16 A and B");
    if (ilv && (dual || lt)) return fail(FG_ERR_UNSUPPORTED, "interleaved complex products take no transforms and are not dual");
    const bool cplx = ilv || (A->im != nullptr) || (B->im != nullptr);
    if (dual && !cplx) return fail(FG_ERR_NULL, "a dual-number product needs the dual planes (im) of A and B");
    if (bf16 && (cplx || A->layout == FG_DIAG || B->layout == FG_DIAG))
        return fail(FG_ERR_UNSUPPORTED, "FG_BF16 operands are supported for real, non-diagonal matrices only");
    if (fg_status st = check_output_matrix("D", D, M, N, cplx)) return st;
    const bool cd16 = D->dtype == FG_F16;
    if (cd16 && (cplx || bf16 || A->layout == FG_DIAG || B->layout == FG_DIAG))
        return fail(FG_ERR_UNSUPPORTED, "FG_F16 C and D are supported for real FG_F16 products in FG_COL or FG_ROW layout");
    const bool has_c = C && C->layout != FG_ZERO && C->re != nullptr;
    if (C && C->layout != FG_ZERO && !C->re && M > 0 && N > 0) return fail(FG_ERR_NULL, "C->re is NULL (pass C == NULL or FG_ZERO for no C term)");
    if (has_c) {
        if (fg_status st = check_output_matrix("C", C, M, N, cplx)) return st;
        if (C->layout != D->layout) return fail(FG_ERR_LAYOUT, "C and D must have the same layout");
        if ((C->dtype == FG_F16) != cd16) return fail(FG_ERR_UNSUPPORTED, "C and D must have the same element type");
    }
    if (A->layout == FG_DIAG && B->layout == FG_DIAG) return fail(FG_ERR_UNSUPPORTED, "at most one of A and B may be diagonal");
    const bool has_ep = ep && (ep->bias || ep->act != FG_ACT_NONE);
    if (ep) {
        if (ep->act != FG_ACT_NONE && ep->act != FG_ACT_RELU) return fail(FG_ERR_LAYOUT, "unknown activation %d", ep->act);
        if (ep->bias && ep->bias_dim != 0 && ep->bias_dim != 1) return fail(FG_ERR_LAYOUT, "bias_dim must be 0 or 1");
        if (ep->bias && !aligned_to(ep->bias, 4)) return fail(FG_ERR_ALIGN, "bias must be aligned to an element");
    }
    if (cplx && has_ep) return fail(FG_ERR_UNSUPPORTED, "bias and activation are not defined for complex or dual products");
    if (cplx && !ilv && (!A->im || !B->im)) return fail(FG_ERR_UNSUPPORTED, "complex and dual products need the second plane of both A and B");
    if (cplx && (A->layout == FG_DIAG || B->layout == FG_DIAG)) return fail(FG_ERR_UNSUPPORTED, "complex or dual diagonal operands are not supported");

    // transforms on loaded elements
    uint16_t a_add = 0, b_add = 0;
    int c_act = FG_ACT_NONE;
    if (lt) {
        if (lt->c_act != FG_ACT_NONE && lt->c_act != FG_ACT_RELU) return fail(FG_ERR_LAYOUT, "unknown activation %d on C", lt->c_act);
        if (!(lt->a_add == lt->a_add) || !(lt->b_add == lt->b_add)) return fail(FG_ERR_SHAPE, "a_add or b_add is NaN");
        const _Float16 ha = (_Float16)lt->a_add, hb = (_Float16)lt->b_add;     // round to nearest even
        memcpy(&a_add, &ha, 2); memcpy(&b_add, &hb, 2);
        if ((a_add & 0x7fff) == 0) a_add = 0;                                   // -0 adds nothing either
        if ((b_add & 0x7fff) == 0) b_add = 0;
        c_act = lt->c_act;
    }
    const bool ab_add = a_add != 0 || b_add != 0;
    if (ab_add && (cplx || bf16 || cd16 || A->layout == FG_DIAG || B->layout == FG_DIAG))
        return fail(FG_ERR_UNSUPPORTED, "an addition on A and B needs real FG_F16 operands in FG_COL or FG_ROW layout and FP32 C and D");
    if (c_act != FG_ACT_NONE && cplx) return fail(FG_ERR_UNSUPPORTED, "an activation on C is not defined for complex or dual products");

    const bool swap = (D->layout == FG_ROW);
    q.cplx = cplx;
    q.cd16 = cd16;
    q.ilv = ilv;
    q.c_act = c_act;
    q.ab_add = ab_add;
    q.a_add = swap ? b_add : a_add;
    q.b_add = swap ? a_add : b_add;
    q.dual = dual;
    q.bf16 = bf16;
    q.alpha = alpha;
    // beta == 0: C is validated but never read (the BLAS convention), so that D may alias an
    // uninitialised C without its NaNs or infinities reaching the result as 0 * x
    const bool use_c = has_c && beta != 0.f;
    q.beta = use_c ? beta : 0.f;
    q.C = use_c ? (const float *)C->re : nullptr;
    q.C_im = use_c ? (const float *)C->im : nullptr;
    q.ldc = use_c ? C->ld : 0;
    q.D = (float *)D->re;
    q.D_im = (float *)D->im;
    q.ldd = D->ld;
    q.bias = (ep && ep->bias) ? ep->bias : nullptr;
    q.bias_dim = ep ? ep->bias_dim : 0;
    q.act = ep ? ep->act : FG_ACT_NONE;
    if (!swap) {
        q.M = M; q.N = N; q.K = K;
        q.A = A->re; q.A_im = A->im; q.lda = A->ld; q.a_diag = A->layout == FG_DIAG; q.a_kc = (A->layout == FG_ROW);
        q.B = B->re; q.B_im = B->im; q.ldb = B->ld; q.b_diag = B->layout == FG_DIAG; q.b_kc = (B->layout == FG_COL);
    } else {
        // D^T (N x M, column-major) = B^T (N x K) . A^T (K x M)
        q.M = N; q.N = M; q.K = K;
        q.A = B->re; q.A_im = B->im; q.lda = B->ld; q.a_diag = B->layout == FG_DIAG; q.a_kc = (B->layout == FG_COL);
        q.B = A->re; q.B_im = A->im; q.ldb = A->ld; q.b_diag = A->layout == FG_DIAG; q.b_kc = (A->layout == FG_ROW);
        q.bias_dim = 1 - q.bias_dim;
    }
    if (q.a_diag) q.a_kc = true;     // a diagonal operand is synthesised K-contiguous in LDS
    if (q.b_diag) q.b_kc = true;
    q.general = false;
    if (g_relaxed.status != FG_OK) {
        if (cplx || q.a_diag || q.b_diag) return fail(g_relaxed.status, "%s (complex, dual and diagonal products have no general kernel)", g_relaxed.msg);
        if (cd16) return fail(g_relaxed.status, "%s (products with FG_F16 C and D have no general kernel)", g_relaxed.msg);
        q.general = true;
    }
    return FG_OK;
}


// ---- tensor contraction -> GEMM description (Section 5.5) -----------------------------------------
// Modes shared by A and C become GEMM rows (M), modes shared by B and C columns (N), modes
// shared by A and B the summed index (K).  Inside a merged index the first mode is the fastest
// (the (ba) -> m convention of the paper's layout listing).  No data moves: the kernel computes
// element offsets from these groups while it loads tiles and stores results.
struct Contraction {
    bool general;            // a requirement of the tiled kernels is missed: use the general kernel
    char why_general[160];
    int64_t M, N, K, batches;
    fg::ModeGroup a_b, b_b, c_b;
    const void *A, *B;
    bool a_kc, b_kc;
    fg::ModeGroup a_m, a_k, b_n, b_k, c_m, c_n;
};

struct TensorView { int32_t n; const int32_t *modes; const int64_t *strides; };

int find_mode(const TensorView &t, int32_t label) {
    for (int i = 0; i < t.n; ++i) if (t.modes[i] == label) return i;
    return -1;
}

fg_status plan_contraction(int32_t nA, const int32_t *modesA, const int64_t *stridesA, const void *A,
                           int32_t nB, const int32_t *modesB, const int64_t *stridesB, const void *B,
                           int32_t nC, const int32_t *modesC, const int64_t *stridesC, const float *Cin, float *Cout,
                           int32_t n_modes, const int32_t *labels, const int64_t *extents, Contraction &c) {
    (void)Cin;
    if (nA < 0 || nB < 0 || nC < 0 || n_modes < 0) return fail(FG_ERR_SHAPE, "negative mode count");
    if ((nA && (!modesA || !stridesA)) || (nB && (!modesB || !stridesB)) || (nC && (!modesC || !stridesC)) || (n_modes && (!labels || !extents)))
        return fail(FG_ERR_NULL, "a mode, stride, label or extent array is NULL");
    if (nA > 12 || nB > 12 || nC > 12 || n_modes > 24) return fail(FG_ERR_UNSUPPORTED, "too many modes");
    TensorView ta{nA, modesA, stridesA}, tb{nB, modesB, stridesB}, tc{nC, modesC, stridesC};
    auto extent_of = [&](int32_t label, int64_t &e) {
        for (int i = 0; i < n_modes; ++i) if (labels[i] == label) { e = extents[i]; return true; }
        return false;
    };
    for (int i = 0; i < n_modes; ++i) {
        if (extents[i] < 0) return fail(FG_ERR_SHAPE, "mode %d has a negative extent", labels[i]);
        for (int j = i + 1; j < n_modes; ++j) if (labels[i] == labels[j]) return fail(FG_ERR_MODES, "mode label %d is listed twice", labels[i]);
    }
    const TensorView *views[3] = {&ta, &tb, &tc};
    const char *names = "ABC";
    for (int v = 0; v < 3; ++v)
        for (int i = 0; i < views[v]->n; ++i) {
            int64_t e;
            if (!extent_of(views[v]->modes[i], e)) return fail(FG_ERR_MODES, "%c uses mode %d, which has no extent", names[v], views[v]->modes[i]);
            for (int j = i + 1; j < views[v]->n; ++j)
                if (views[v]->modes[i] == views[v]->modes[j]) return fail(FG_ERR_MODES, "%c lists mode %d twice (trace modes are not supported)", names[v], views[v]->modes[i]);
        }
    // every used label must sit in exactly two tensors
    bool any_zero = false;
    for (int i = 0; i < n_modes; ++i) {
        int cnt = (find_mode(ta, labels[i]) >= 0) + (find_mode(tb, labels[i]) >= 0) + (find_mode(tc, labels[i]) >= 0);
        if (cnt == 0) continue;
        if (cnt == 1) return fail(FG_ERR_MODES, "mode %d appears in only one of A, B, C (no reduction or broadcast modes)", labels[i]);
        if (extents[i] == 0) any_zero = true;
    }
    c.M = c.N = 0; c.K = 0; c.batches = 1;
    c.general = false; c.why_general[0] = 0;
    if (any_zero) return FG_OK;               // an empty tensor: nothing to compute
    if (!A || !B || !Cout) return fail(FG_ERR_NULL, "A, B or Cout is NULL");
    if (!aligned_to(A, 2) || !aligned_to(B, 2) || !aligned_to(Cout, 4) || (Cin && !aligned_to(Cin, 4)))
        return fail(FG_ERR_ALIGN, "tensor base pointers must be aligned to an element");
    // A description that misses a requirement of the tiled kernels is computed by the general
    // kernel; the first reason is kept for fg_contract_plan.
    auto need_general = [&](const char *fmt, int x = 0, int y = 0) {
        if (!c.general) { c.general = true; snprintf(c.why_general, sizeof c.why_general, fmt, x, y); }
    };
    if (!aligned16(A) || !aligned16(B) || !aligned16(Cout) || (Cin && !aligned16(Cin))) need_general("a tensor base pointer is not 16-byte aligned");

    // Lanes of the result run along GEMM rows, so C's unit-stride mode should be a row mode:
    // exchange the roles of A and B when it belongs to B only.
    int c_unit = -1;
    for (int i = 0; i < nC; ++i) { int64_t e; extent_of(modesC[i], e); if (stridesC[i] == 1 && e > 1) { c_unit = modesC[i]; break; } }
    if (c_unit >= 0 && find_mode(tb, c_unit) >= 0 && find_mode(ta, c_unit) < 0) { TensorView t = ta; ta = tb; tb = t; const void *q = A; A = B; B = q; }
    c.A = A; c.B = B;
    auto in_a = [&](int32_t l) { return find_mode(ta, l) >= 0; };
    auto in_b = [&](int32_t l) { return find_mode(tb, l) >= 0; };
    auto in_c = [&](int32_t l) { return find_mode(tc, l) >= 0; };
    auto is_row = [&](int32_t l) { return in_a(l) && in_c(l) && !in_b(l); };
    auto is_col = [&](int32_t l) { return in_b(l) && in_c(l) && !in_a(l); };
    auto is_sum = [&](int32_t l) { return in_a(l) && in_b(l) && !in_c(l); };
    auto is_batch = [&](int32_t l) { return in_a(l) && in_b(l) && in_c(l); };

    auto unit_mode = [&](const TensorView &t) {
        int best = -1;
        for (int i = 0; i < t.n; ++i) {
            int64_t e; extent_of(t.modes[i], e);
            if (t.strides[i] == 1 && e % 8 == 0 && e > 0 && !is_batch(t.modes[i])) { best = t.modes[i]; break; }
        }
        return best;
    };
    int ua = unit_mode(ta), ub = unit_mode(tb);
    if (ua < 0 || ub < 0) need_general("A or B has no row, column or summed mode with stride 1 and an extent that is a multiple of 8");
    c.a_kc = ua >= 0 && is_sum(ua);           // A's contiguous mode is summed over
    c.b_kc = ub >= 0 && is_sum(ub);
    if (c.a_kc && c.b_kc && ua != ub) need_general("A and B are contiguous along different summed modes (%d and %d)", ua, ub);
    if (c.general) { ua = ub = -1; c.a_kc = c.b_kc = false; }   // the merged indices then follow the tensors' own mode order

    // order of the modes inside each merged index
    int32_t m_modes[16], n_modes_[16], k_modes[16], b_modes[16];
    int nm = 0, nn = 0, nkk = 0, nb = 0;
    auto push_unique = [](int32_t *arr, int &n, int32_t label) { for (int i = 0; i < n; ++i) if (arr[i] == label) return; arr[n++] = label; };
    if (!c.a_kc && ua >= 0) push_unique(m_modes, nm, ua);
    else if (c_unit >= 0 && is_row(c_unit)) push_unique(m_modes, nm, c_unit);
    for (int i = 0; i < tc.n; ++i) if (is_row(tc.modes[i])) push_unique(m_modes, nm, tc.modes[i]);
    if (!c.b_kc && ub >= 0) push_unique(n_modes_, nn, ub);
    for (int i = 0; i < tc.n; ++i) if (is_col(tc.modes[i])) push_unique(n_modes_, nn, tc.modes[i]);
    if (c.a_kc) push_unique(k_modes, nkk, ua);
    else if (c.b_kc) push_unique(k_modes, nkk, ub);
    for (int i = 0; i < ta.n; ++i) if (is_sum(ta.modes[i])) push_unique(k_modes, nkk, ta.modes[i]);
    for (int i = 0; i < tc.n; ++i) if (is_batch(tc.modes[i])) push_unique(b_modes, nb, tc.modes[i]);
    if (nm > fg::kMaxGroupModes || nn > fg::kMaxGroupModes || nkk > fg::kMaxGroupModes || nb > fg::kMaxGroupModes)
        return fail(FG_ERR_UNSUPPORTED, "at most %d modes per merged index", fg::kMaxGroupModes);
    if (nkk == 0) need_general("no summed mode (an outer product)");

    // Modes of extent 1 carry no index and are dropped.  For the others the kernel divides by the
    // extent with a multiply-high: with 2^s < e <= 2^(s+1) and magic = floor(2^(32+s)/e) + 1,
    // floor(idx / e) == (idx * magic) >> (32 + s) for every 0 <= idx < 2^31.
    auto fill = [&](fg::ModeGroup &g, const int32_t *modes, int n, const TensorView &t, int64_t &total) {
        g.n = 0; total = 1;
        for (int i = 0; i < n; ++i) {
            int64_t e; extent_of(modes[i], e);
            total *= e;
            if (e == 1) continue;
            int k = g.n++;
            g.extent[k] = (int32_t)e;
            g.stride[k] = t.strides[find_mode(t, modes[i])];
            uint32_t sh = 0;
            while ((2ull << sh) < (uint64_t)e) ++sh;          // 2^sh < e <= 2^(sh+1)
            g.shift[k] = sh;
            g.magic[k] = (uint32_t)(((1ull << (32 + sh)) / (uint64_t)e) + 1);
        }
        for (int i = g.n; i < fg::kMaxGroupModes; ++i) { g.extent[i] = 2; g.stride[i] = 0; g.magic[i] = 0; g.shift[i] = 0; }
    };
    int64_t t1, t2;
    fill(c.a_m, m_modes, nm, ta, c.M); fill(c.c_m, m_modes, nm, tc, t1);
    fill(c.b_n, n_modes_, nn, tb, c.N); fill(c.c_n, n_modes_, nn, tc, t2);
    fill(c.a_k, k_modes, nkk, ta, c.K); fill(c.b_k, k_modes, nkk, tb, t1);
    fill(c.a_b, b_modes, nb, ta, c.batches); fill(c.b_b, b_modes, nb, tb, t1); fill(c.c_b, b_modes, nb, tc, t2);
    if (nb == 0) c.batches = 1;
    if (nm == 0) c.M = 1;
    if (nn == 0) c.N = 1;

    for (int i = 0; i < ta.n; ++i) if (ta.strides[i] < 0) return fail(FG_ERR_UNSUPPORTED, "negative strides are not supported");
    for (int i = 0; i < tb.n; ++i) if (tb.strides[i] < 0) return fail(FG_ERR_UNSUPPORTED, "negative strides are not supported");
    for (int i = 0; i < tc.n; ++i) if (tc.strides[i] < 0) return fail(FG_ERR_UNSUPPORTED, "negative strides are not supported");
    if (!c.general) {
        if ((c.a_kc || c.b_kc) && c.a_k.n > 0 && c.a_k.extent[0] % 8) need_general("the leading summed mode (%d) is contiguous in A or B and its extent is not a multiple of 8", k_modes[0]);
        if (c.a_kc && c.a_k.n > 0 && c.a_k.stride[0] != 1) need_general("the leading summed mode is not contiguous in A");
        if (c.b_kc && c.b_k.n > 0 && c.b_k.stride[0] != 1) need_general("the leading summed mode (%d) is contiguous in A but not in B", k_modes[0]);
        if ((c.a_kc || c.b_kc) && c.a_k.n == 0) need_general("the contiguous summed mode has extent 1");
        if (!c.a_kc && (c.a_m.n == 0 || c.a_m.stride[0] != 1 || c.a_m.extent[0] % 8)) need_general("A's contiguous row mode must have an extent that is a multiple of 8");
        if (!c.b_kc && (c.b_n.n == 0 || c.b_n.stride[0] != 1 || c.b_n.extent[0] % 8)) need_general("B's contiguous column mode must have an extent that is a multiple of 8");
        // The tiled kernels fetch 16-byte pieces along the contiguous mode: every other stride of A
        // and B must keep those pieces 16-byte aligned.
        auto strides_ok = [](const fg::ModeGroup &g, int first) {
            for (int t = first; t < g.n; ++t) if (g.stride[t] % 8) return false;
            return true;
        };
        if (!strides_ok(c.a_m, c.a_kc ? 0 : 1) || !strides_ok(c.a_k, c.a_kc ? 1 : 0) || !strides_ok(c.a_b, 0))
            need_general("a stride of A other than its contiguous mode's is not a multiple of 8 elements");
        if (!strides_ok(c.b_n, c.b_kc ? 0 : 1) || !strides_ok(c.b_k, c.b_kc ? 1 : 0) || !strides_ok(c.b_b, 0))
            need_general("a stride of B other than its contiguous mode's is not a multiple of 8 elements");
        // the tiled kernels address A, B and C with 32-bit byte offsets inside a 2 GiB window
        auto span = [&](const TensorView &t) {
            int64_t sp = 1;
            for (int i = 0; i < t.n; ++i) { int64_t e; extent_of(t.modes[i], e); sp += (e - 1) * t.strides[i]; }
            return sp;
        };
        if (span(ta) * 2 >= (1ll << 31) || span(tb) * 2 >= (1ll << 31) || span(tc) * 4 >= (1ll << 31)) need_general("A, B or C spans 2 GiB or more");
    }
    if (!c.general) {
        if (c.a_k.n == 0) {
            // every summed mode has extent 1: one K step whose k = 0 alone is loaded
            c.a_k.n = c.b_k.n = 1;
            c.a_k.extent[0] = c.b_k.extent[0] = 1;
            c.a_k.stride[0] = c.b_k.stride[0] = 0;
        }
        // K steps of 64 walk the leading summed mode; when its extent is not a multiple of 64 the
        // last step of each pass is zero-filled, so the tiled kernels see that extent rounded up
        c.K = c.K / c.a_k.extent[0] * ((c.a_k.extent[0] + 63) / 64 * 64);
    }
    if (c.M > (1 << 30) || c.N > (1 << 30) || c.K > (1 << 30) || c.batches > (1 << 20)) return fail(FG_ERR_UNSUPPORTED, "merged extents above 2^30 (2^20 for batch modes) are not supported");
    return FG_OK;
}

}  // namespace

extern "C" {

const char *fg_last_error(void) { return g_err; }

int32_t fg_version(void) { return 100; }   // 0.1.0

fg_status fg_init(void) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FG_ERR_LAUNCH, "no HIP device is current");
    struct { const fg::KernelEntry *t; int n; } tables[] = {
        {fg::kernel_table_nn(), fg::TILE_COUNT * fg::VARIANT_COUNT}, {fg::kernel_table_nt(), fg::TILE_COUNT * fg::VARIANT_COUNT},
        {fg::kernel_table_tn(), fg::TILE_COUNT * fg::VARIANT_COUNT}, {fg::kernel_table_tt(), fg::TILE_COUNT * fg::VARIANT_COUNT},
        {fg::kernel_table_nn_bf16(), fg::TILE_COUNT}, {fg::kernel_table_nt_bf16(), fg::TILE_COUNT},
        {fg::kernel_table_tn_bf16(), fg::TILE_COUNT}, {fg::kernel_table_tt_bf16(), fg::TILE_COUNT},
        {fg::kernel_table_nn_xf(), fg::TILE_COUNT}, {fg::kernel_table_nt_xf(), fg::TILE_COUNT},
        {fg::kernel_table_tn_xf(), fg::TILE_COUNT}, {fg::kernel_table_tt_xf(), fg::TILE_COUNT},
        {fg::kernel_table_nn_h16(), fg::TILE_COUNT}, {fg::kernel_table_nt_h16(), fg::TILE_COUNT},
        {fg::kernel_table_tn_h16(), fg::TILE_COUNT}, {fg::kernel_table_tt_h16(), fg::TILE_COUNT},
        {fg::kernel_table_diag(), fg::DIAG_TILE_COUNT * 4},
        {fg::kernel_table_cplx(), fg::CTILE_COUNT * 4}, {fg::kernel_table_dual(), fg::CTILE_COUNT * 4},
        {fg::kernel_table_cplx_il(), fg::CTILE_COUNT * 4},
    };
    for (auto &tb : tables)
        for (int i = 0; i < tb.n; ++i) {
            int per_cu = 0;
            if (!tb.t[i].fn) continue;          // a variant that is not built for this tile
            if (fg_status st = prepare(tb.t[i], dev, per_cu)) return st;
        }
    float *st = nullptr;
    if (fg_status s2 = static_scratch(dev, &st)) return s2;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    Workspace *w = nullptr;
    return workspace_locked(dev, nullptr, true, &w);
}

// static_only: the allocation-free entry point.  Same plan as the ordinary call; partial products
// of a K split go to the static scratch array (FG_ERR_UNSUPPORTED if they do not fit), and nothing
// on this path allocates, frees or creates anything.
static fg_status gemm_impl(int64_t M, int64_t N, int64_t K, float alpha, const fg_matrix *A, const fg_matrix *B,
                           float beta, const fg_matrix *C, const fg_matrix *D, const fg_epilogue *ep, bool dual,
                           const fg_load_transforms *lt, void *hip_stream, bool static_only = false) {
    Problem q;
    if (fg_status st = normalise(M, N, K, alpha, A, B, beta, C, D, ep, dual, lt, q)) return st;
    if (q.M == 0 || q.N == 0) return FG_OK;
    if (q.general) {
        fg::FallbackParams f;
        memset(&f, 0, sizeof f);
        f.M = (int32_t)q.M; f.N = (int32_t)q.N; f.K = (int32_t)q.K;
        f.A = (const uint16_t *)q.A; f.B = (const uint16_t *)q.B;
        f.a_rs = q.a_kc ? q.lda : 1; f.a_ks = q.a_kc ? 1 : q.lda;
        f.b_rs = q.b_kc ? q.ldb : 1; f.b_ks = q.b_kc ? 1 : q.ldb;
        f.C = q.C; f.D = q.D; f.ldc = q.ldc; f.ldd = q.ldd;
        f.bias = q.bias; f.bias_dim = q.bias_dim; f.act = q.act; f.c_act = q.c_act;
        f.alpha = q.alpha; f.beta = q.beta;
        f.a_add = q.a_add; f.b_add = q.b_add; f.ab_add = q.ab_add; f.bf16 = q.bf16;
        if ((int64_t)((q.M + 63) / 64) * ((q.N + 63) / 64) >= (1ll << 31)) return fail(FG_ERR_UNSUPPORTED, "too many tiles");
        hipError_t e = fg::launch_gemm_fallback(f, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "launch of the general kernel failed: %s", hipGetErrorString(e));
        return FG_OK;
    }
    Plan plan{0, 1, 1};
    const fg::KernelEntry *kp = select_kernel(q, &plan);
    if (!kp) return fail(FG_ERR_UNSUPPORTED, "no kernel for M=%lld, N=%lld", (long long)q.M, (long long)q.N);
    const fg::KernelEntry &k = *kp;

    fg::GemmParams p;
    memset(&p, 0, sizeof p);
    p.M = (int32_t)q.M; p.N = (int32_t)q.N; p.K = (int32_t)q.K;
    p.tiles_m = (int32_t)((q.M + k.bm - 1) / k.bm); p.tiles_n = (int32_t)((q.N + k.bn - 1) / k.bn);
    p.A = (const _Float16 *)q.A; p.B = (const _Float16 *)q.B;
    p.A_im = (const _Float16 *)q.A_im; p.B_im = (const _Float16 *)q.B_im;
    p.a_rs = q.a_kc ? q.lda : 1; p.a_ks = q.a_kc ? 1 : q.lda;
    p.b_rs = q.b_kc ? q.ldb : 1; p.b_ks = q.b_kc ? 1 : q.ldb;
    // stored span of each operand, rounded up to whole 16-byte chunks (see TileLoader::begin)
    auto span8 = [](bool kc, int64_t rows, int64_t k, int64_t ld) { int64_t s = kc ? (rows - 1) * ld + k : (k - 1) * ld + rows; return (s + 7) / 8 * 8; };
    p.a_span = q.K > 0 ? span8(q.a_kc, q.M, q.K, q.lda) : 0;
    p.b_span = q.K > 0 ? span8(q.b_kc, q.N, q.K, q.ldb) : 0;
    // A and B may be of any size; what must fit 32 bits is the byte offset a lane forms inside one
    // block panel at one K step (up to 256 rows by 64 k) and the advance from one K step to the next.
    const int64_t ab_elem_bytes = q.ilv ? 4 : 2;
    auto reach = [&](bool kc, int64_t ld) { return (kc ? 255 * ld + 64 : 64 * ld + 256) * ab_elem_bytes; };
    if ((!q.a_diag && reach(q.a_kc, q.lda) >= (1ll << 31)) || (!q.b_diag && reach(q.b_kc, q.ldb) >= (1ll << 31)))
        return fail(FG_ERR_UNSUPPORTED, "leading dimension of A or B too large (row-of-K operands: below 2^22 elements, others below 2^24)");
    const int64_t cd_limit = q.ilv ? (1ll << 20) : (1ll << 21);
    if (q.ldc >= cd_limit || q.ldd >= cd_limit) return fail(FG_ERR_UNSUPPORTED, "leading dimension of C or D must be below 2^21 elements (2^20 interleaved)");
    p.C = q.C; p.D = q.D; p.C_im = q.C_im; p.D_im = q.D_im; p.ldc = q.ldc; p.ldd = q.ldd;
    p.bias = q.bias; p.bias_dim = q.bias_dim; p.act = q.act; p.has_c = q.C != nullptr;
    p.c_act = q.c_act;
    p.a_add2 = (uint32_t)q.a_add * 0x10001u; p.b_add2 = (uint32_t)q.b_add * 0x10001u;
    p.alpha = q.alpha; p.beta = q.beta;
    const int64_t tiles64 = (int64_t)p.tiles_m * p.tiles_n;
    if (tiles64 >= (1ll << 31) / 64) return fail(FG_ERR_UNSUPPORTED, "too many tiles");
    const int tiles = (int)tiles64;
    p.tile_begin = 0; p.tile_count = tiles; p.splits = 1;
    {
        // C and D stream past the L2 (they are touched once and would displace the A and B panels that
        // other workgroups re-read), unless the whole problem fits the 256 MB memory-side cache: then
        // nothing is displaced for long, and keeping C and D cached measured faster (3000^3: 73.6
        // against 87.4 us, 4096^3: -6 %, 5000 x 3000 x 2000: 76.7 against 103.1 us back to back;
        // equal on cache-cold operands; from 300 MB up streaming wins by 4 to 9 %).
        const int64_t es_cd = q.cd16 ? 2 : 4;
        const int64_t bytes = (q.M * q.K + q.K * q.N) * 2 + q.M * q.N * es_cd * (q.C ? 2 : 1);
        p.cd_cached = bytes <= (256ll << 20);
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    if (plan.splits <= 1 && plan.tail_splits <= 1) return launch(k, p, stream);

    // Split K for all tiles, or for the tiles of the last round only: partial products into the
    // workspace, then the reduction pass that also applies alpha, beta.C, bias and the activations.
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FG_ERR_LAUNCH, "no HIP device is current");
    int S = plan.splits, first = 0, count = tiles;
    if (plan.tail_splits > 1) {
        int per_cu = 0;
        if (fg_status st = prepare(k, dev, per_cu)) return st;
        const int slots = per_cu * kNumCU;
        first = tiles / slots * slots; count = tiles - first; S = plan.tail_splits;
        if (first == 0 || count == 0 || (int64_t)count * S * k.bm * k.bn * 4 > kWorkspaceBytes) S = 1;
    }
    if (S == 1) return launch(k, p, stream);
    const int64_t need = (int64_t)count * S * k.bm * k.bn * 4;
    float *ws = nullptr;
    Workspace *guard = nullptr;
    std::unique_lock<std::mutex> ws_lock(g_ws_mutex, std::defer_lock);
    if (static_only) {
        if (need > kStaticScratchBytes)
            return fail(FG_ERR_UNSUPPORTED, "this problem is computed as %d partial products over K, which need %lld bytes of scratch memory; the "
                                            "static scratch array of the allocation-free entry point holds %lld (use fg_gemm_ex)",
                        S, (long long)need, (long long)kStaticScratchBytes);
        if (fg_status st = static_scratch(dev, &ws)) return st;
    } else {
        ws_lock.lock();
        if (fg_status st = workspace_locked(dev, stream, true, &guard)) return st;
        ws = guard->ptr;
        if (stream_is_capturing(stream)) guard = nullptr;      // a captured call is ordered by its graph's caller
        else if (guard->used && guard->last_stream != stream) {
            hipError_t e = hipStreamWaitEvent(stream, guard->last_use, 0);
            if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "hipStreamWaitEvent on the workspace's last use failed: %s", hipGetErrorString(e));
        }
    }
    if (first > 0) {
        fg::GemmParams head = p;
        head.tile_count = first;
        if (fg_status st = launch(k, head, stream)) return st;
    }
    const int64_t nk = (q.K + 63) / 64;
    fg::GemmParams part = p;
    part.tile_begin = first; part.tile_count = count;
    part.splits = S;
    part.split_kt = (int32_t)((nk + S - 1) / S);
    part.D = ws;
    part.C = nullptr; part.has_c = 0; part.bias = nullptr; part.act = 0; part.c_act = 0; part.alpha = 1.f; part.beta = 0.f;
    if (fg_status st = launch(k, part, stream)) return st;
    hipError_t e = fg::launch_splitk_reduce(ws, S, first, count, k.bm, k.bn, p.tiles_m, p.tiles_n, (int)q.M, (int)q.N, q.alpha, q.beta,
                                            q.C, q.ldc, q.D, q.ldd, q.bias, q.bias_dim, q.act, q.c_act, stream);
    if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "launch of the split-K reduction failed: %s", hipGetErrorString(e));
    if (guard) {
        e = hipEventRecord(guard->last_use, stream);
        if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "hipEventRecord after the split-K reduction failed: %s", hipGetErrorString(e));
        guard->last_stream = stream;
        guard->used = true;
    }
    return FG_OK;
}

fg_status fg_gemm(int64_t M, int64_t N, int64_t K, float alpha, const fg_matrix *A, const fg_matrix *B,
                  float beta, const fg_matrix *C, const fg_matrix *D, const fg_epilogue *ep, void *hip_stream) {
    return gemm_impl(M, N, K, alpha, A, B, beta, C, D, ep, false, nullptr, hip_stream);
}

fg_status fg_gemm_ex(int64_t M, int64_t N, int64_t K, float alpha, const fg_matrix *A, const fg_matrix *B,
                     float beta, const fg_matrix *C, const fg_matrix *D, const fg_epilogue *ep,
                     const fg_load_transforms *lt, void *hip_stream) {
    return gemm_impl(M, N, K, alpha, A, B, beta, C, D, ep, false, lt, hip_stream);
}

fg_status fg_gemm_noalloc(int64_t M, int64_t N, int64_t K, float alpha, const fg_matrix *A, const fg_matrix *B,
                          float beta, const fg_matrix *C, const fg_matrix *D, const fg_epilogue *ep,
                          const fg_load_transforms *lt, void *hip_stream) {
    return gemm_impl(M, N, K, alpha, A, B, beta, C, D, ep, false, lt, hip_stream, true);
}

void fg_reload_tuning(void) { read_tuning_from_environment(); }

fg_status fg_gemm_dual(int64_t M, int64_t N, int64_t K, float alpha, const fg_matrix *A, const fg_matrix *B,
                       float beta, const fg_matrix *C, const fg_matrix *D, void *hip_stream) {
    return gemm_impl(M, N, K, alpha, A, B, beta, C, D, nullptr, true, nullptr, hip_stream);
}

fg_status fg_gemm_plan(int64_t M, int64_t N, int64_t K, int32_t layoutA, int32_t layoutB, int32_t layoutD,
                       int32_t variant, char *buf, int32_t buf_len) {
    if (!buf || buf_len <= 0) return fail(FG_ERR_NULL, "buf is NULL or empty");
    buf[0] = 0;
    g_relaxed.status = FG_OK;
    if (fg_status st = check_sizes(M, N, K)) return st;
    auto ok_in = [](int32_t l) { return l == FG_COL || l == FG_ROW || l == FG_DIAG; };
    if (!ok_in(layoutA) || !ok_in(layoutB) || (layoutD != FG_COL && layoutD != FG_ROW))
        return fail(FG_ERR_LAYOUT, "plan query: A, B take FG_COL / FG_ROW / FG_DIAG, D takes FG_COL / FG_ROW");
    if (layoutA == FG_DIAG && layoutB == FG_DIAG) return fail(FG_ERR_UNSUPPORTED, "at most one of A and B may be diagonal");
    if (variant < FG_PLAN_REAL || variant > FG_PLAN_REAL_AB_ADD) return fail(FG_ERR_LAYOUT, "plan query: unknown variant %d", variant);
    if (variant != FG_PLAN_REAL && (layoutA == FG_DIAG || layoutB == FG_DIAG))
        return fail(FG_ERR_UNSUPPORTED, "diagonal operands are supported for real FG_F16 products only");
    Problem q;
    memset(&q, 0, sizeof q);
    q.cplx = variant == FG_PLAN_COMPLEX || variant == FG_PLAN_DUAL || variant == FG_PLAN_COMPLEX_INTERLEAVED;
    q.ilv = variant == FG_PLAN_COMPLEX_INTERLEAVED;
    q.dual = variant == FG_PLAN_DUAL;
    q.bf16 = variant == FG_PLAN_REAL_BF16;
    q.cd16 = variant == FG_PLAN_REAL_F16_CD;
    q.ab_add = variant == FG_PLAN_REAL_AB_ADD;
    if (layoutD == FG_COL) {
        q.M = M; q.N = N;
        q.a_diag = layoutA == FG_DIAG; q.b_diag = layoutB == FG_DIAG;
        q.a_kc = layoutA == FG_ROW || q.a_diag; q.b_kc = layoutB == FG_COL || q.b_diag;
    } else {
        q.M = N; q.N = M;
        q.a_diag = layoutB == FG_DIAG; q.b_diag = layoutA == FG_DIAG;
        q.a_kc = layoutB == FG_COL || q.a_diag; q.b_kc = layoutA == FG_ROW || q.b_diag;
    }
    q.K = K;
    if (g_relaxed.status != FG_OK) {
        // K is not a multiple of 8 (alignment is not known to this query)
        if (q.cplx || q.a_diag || q.b_diag || q.cd16) return fail(g_relaxed.status, "%s (complex, dual, diagonal and FG_F16-result products have no general kernel)", g_relaxed.msg);
        snprintf(buf, (size_t)buf_len, "gemm_general_64x64x32");
        return FG_OK;
    }
    Plan plan{0, 1, 1};
    const fg::KernelEntry *k = select_kernel(q, &plan);
    if (!k) return fail(FG_ERR_UNSUPPORTED, "no kernel for the problem");
    if (plan.splits > 1) snprintf(buf, (size_t)buf_len, "%s+splitk%d", k->name, plan.splits);
    else if (plan.tail_splits > 1) snprintf(buf, (size_t)buf_len, "%s+tailsplitk%d", k->name, plan.tail_splits);
    else snprintf(buf, (size_t)buf_len, "%s", k->name);
    return FG_OK;
}

// Kernel for a planned contraction (tiled kernels only): tile shape, streaming variant, row order.
static const fg::KernelEntry *select_contract_kernel(const Contraction &c, const float *Cin, const float *Cout, int *perm_z_out) {
    // A result that is not contiguous along the leading row mode is stored in short pieces; the
    // smallest tile makes them shorter still (measured on the paper's D_abc = A_bda B_dc).
    const bool rows_contiguous = c.c_m.n == 0 || c.c_m.stride[0] == 1;
    const int tile = choose_plan(c.M, c.N, c.K, false, rows_contiguous || c.M < 128 || c.N < 128, c.batches, true).tile;
    // The result streams past the L2 only if every store of 32 consecutive rows is one whole,
    // aligned 128-byte line: leading row mode contiguous with an extent that is a multiple of 32,
    // every other stride of C and its base a multiple of 32 elements.
    auto whole_lines = [](const fg::ModeGroup &g, int first) {
        for (int t = first; t < g.n; ++t) if (g.stride[t] % 32) return false;
        return true;
    };
    const bool c_stream = c.c_m.n > 0 && c.c_m.stride[0] == 1 && c.c_m.extent[0] % 32 == 0 && whole_lines(c.c_m, 1) &&
                          whole_lines(c.c_n, 0) && whole_lines(c.c_b, 0) && (uintptr_t)Cout % 128 == 0 &&
                          (!Cin || (uintptr_t)Cin % 128 == 0);
    const fg::KernelEntry &k = table_for(c.a_kc, c.b_kc)[fg::entry_index(tile, c_stream ? fg::VARIANT_CONTRACT_STREAM : fg::VARIANT_CONTRACT)];
    // Row order inside a tile (tile_row in the kernel): when A is contiguous along its leading row
    // mode but C along the next one, and the leading mode is short enough that a tile spans at
    // least four values of the next, let every accumulator hold 8 x 4 of (leading, next).
    *perm_z_out = 1;
    if (k.fn && !c.a_kc && c.c_m.n >= 2 && c.c_m.stride[1] == 1) {
        const int e0 = c.a_m.extent[0];
        if (e0 % 8 == 0 && k.bm % e0 == 0 && k.bm / e0 >= 4) *perm_z_out = k.bm / e0;
    }
    return k.fn ? &k : nullptr;
}

fg_status fg_contract(int32_t nA, const int32_t *modesA, const int64_t *stridesA, const void *A,
                      int32_t nB, const int32_t *modesB, const int64_t *stridesB, const void *B,
                      int32_t nC, const int32_t *modesC, const int64_t *stridesC, const float *Cin, float *Cout,
                      int32_t n_modes, const int32_t *mode_labels, const int64_t *mode_extents,
                      float alpha, float beta, void *hip_stream) {
    Contraction c;
    if (fg_status st = plan_contraction(nA, modesA, stridesA, A, nB, modesB, stridesB, B, nC, modesC, stridesC,
                                        Cin, Cout, n_modes, mode_labels, mode_extents, c))
        return st;
    if (c.M == 0 || c.N == 0) return FG_OK;
    const bool use_c = Cin != nullptr && beta != 0.f;        // beta == 0: Cin is never read
    if (c.general) {
        fg::ContractFallbackParams f;
        memset(&f, 0, sizeof f);
        f.M = (int32_t)c.M; f.N = (int32_t)c.N; f.K = (int32_t)c.K; f.batches = (int32_t)c.batches;
        f.A = (const _Float16 *)c.A; f.B = (const _Float16 *)c.B;
        f.C = use_c ? Cin : nullptr; f.D = Cout;
        f.a_m = c.a_m; f.a_k = c.a_k; f.b_n = c.b_n; f.b_k = c.b_k; f.c_m = c.c_m; f.c_n = c.c_n;
        f.a_b = c.a_b; f.b_b = c.b_b; f.c_b = c.c_b;
        f.alpha = alpha; f.beta = use_c ? beta : 0.f;
        f.a_kfast = c.a_k.n > 0 && c.a_k.stride[0] == 1;
        f.b_kfast = c.b_k.n > 0 && c.b_k.stride[0] == 1;
        if (((c.M + 63) / 64) * ((c.N + 63) / 64) * c.batches >= (1ll << 31)) return fail(FG_ERR_UNSUPPORTED, "too many tiles");
        hipError_t e = fg::launch_contract_fallback(f, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail(FG_ERR_LAUNCH, "launch of the general contraction kernel failed: %s", hipGetErrorString(e));
        return FG_OK;
    }
    int perm_z = 1;
    const fg::KernelEntry *kp = select_contract_kernel(c, Cin, Cout, &perm_z);
    if (!kp) return fail(FG_ERR_UNSUPPORTED, "internal: no contraction kernel for this tile");
    const fg::KernelEntry &k = *kp;
    fg::GemmParams p;
    memset(&p, 0, sizeof p);
    p.M = (int32_t)c.M; p.N = (int32_t)c.N; p.K = (int32_t)c.K;
    p.tiles_m = (int32_t)((c.M + k.bm - 1) / k.bm); p.tiles_n = (int32_t)((c.N + k.bn - 1) / k.bn);
    p.A = (const _Float16 *)c.A; p.B = (const _Float16 *)c.B;
    p.C = use_c ? Cin : nullptr; p.D = Cout;
    p.has_c = use_c;
    p.alpha = alpha; p.beta = use_c ? beta : 0.f;
    p.a_m = c.a_m; p.a_k = c.a_k; p.b_n = c.b_n; p.b_k = c.b_k; p.c_m = c.c_m; p.c_n = c.c_n;
    p.a_b = c.a_b; p.b_b = c.b_b; p.c_b = c.c_b; p.batches = (int32_t)c.batches;
    if ((int64_t)p.tiles_m * p.tiles_n * c.batches >= (1ll << 31)) return fail(FG_ERR_UNSUPPORTED, "too many tiles");
    p.perm_z = perm_z;
    return launch(k, p, (hipStream_t)hip_stream);
}

fg_status fg_contract_plan(int32_t nA, const int32_t *modesA, const int64_t *stridesA, const void *A,
                           int32_t nB, const int32_t *modesB, const int64_t *stridesB, const void *B,
                           int32_t nC, const int32_t *modesC, const int64_t *stridesC, const float *Cin, float *Cout,
                           int32_t n_modes, const int32_t *mode_labels, const int64_t *mode_extents,
                           char *buf, int32_t buf_len) {
    if (!buf || buf_len <= 0) return fail(FG_ERR_NULL, "buf is NULL or empty");
    buf[0] = 0;
    Contraction c;
    if (fg_status st = plan_contraction(nA, modesA, stridesA, A, nB, modesB, stridesB, B, nC, modesC, stridesC,
                                        Cin, Cout, n_modes, mode_labels, mode_extents, c))
        return st;
    if (c.M == 0 || c.N == 0) { snprintf(buf, (size_t)buf_len, "nothing to compute"); return FG_OK; }
    if (c.general) { snprintf(buf, (size_t)buf_len, "gett_general_64x64x32 (%s)", c.why_general); return FG_OK; }
    int perm_z = 1;
    const fg::KernelEntry *k = select_contract_kernel(c, Cin, Cout, &perm_z);
    if (!k) return fail(FG_ERR_UNSUPPORTED, "internal: no contraction kernel for this tile");
    snprintf(buf, (size_t)buf_len, "%s", k->name);
    return FG_OK;
}

}  // extern "C"
