// Vector-LUT ternary x INT8 mpGeMM for MI355X (gfx950): kernels and C ABI.
//
// Data layout in LDS (one "slot" = one 81-row table whose rows are 256 bytes):
//   a 256-byte row is 16 slices of 16 bytes; slice l belongs to LDS banks 4l..4l+3,
//   so 16 lanes that each read "their" slice of 16 different rows never conflict.
//   A slice holds 8 INT16 table entries (8 tokens) of ONE sub-table.  With
//   J = 1,2,4,8,16 sub-tables interleaved per row, a slot serves J sub-tables x
//   (128/J) tokens: slice l = j * (16/J) + t  (j = sub-table selector, t = 8-token chunk).
//   Lane (grp = lane/16, l = lane%16) of a wave looks up row idx of slice l for
//   output row 4*rowgroup + grp, so one ds_read_b128 serves 4 output rows x 128
//   (sub-table, token) pairs; the J partial sums of a token are added across lanes
//   once, after the K loop.
//
// Paper references: Alg. 1 (lookup/accumulate and Precompute), Eq. 1-2, Sec. 3.3
// (token-contiguous tables, tile-contiguous packed weights), Sec. 3.4 (tiling,
// streamed precompute-lookup, INT16->INT32 hierarchy, block size 64), Sec. 4
// (topological precompute).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>

#include "vlut.h"


// The kernels, one header per kernel family; this file holds the host side (launch plans, launches, the C ABI).
#include "common.hip.h"
#include "prepare_kernels.hip.h"
#include "lookup_kernel.hip.h"
#include "mfma_kernel.hip.h"
#include "lookup5_kernel.hip.h"
#include "narrow_kernel.hip.h"
#include "small_kernels.hip.h"

// Scratch of vlut_mpgemm_static (split-K partial sums, INT32 [S][N][M]): device memory owned by the library, one
// copy per GPU, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; every use of the memory goes through the per-device pointer kept below.
static __device__ __align__(256) unsigned char scratch[VLUT_STATIC_SCRATCH_BYTES];

namespace {

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device (with that device current).
int static_scratch_ptr(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VLUT_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return VLUT_ERR_DEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return VLUT_OK;
}

// Raises a kernel's dynamic LDS limit once per device (the limit is a property of the kernel on one device).
// The table kernels form LDS addresses as idx*256 + slice*16 and so need their dynamic LDS segment to start at LDS
// address 0, i.e. a kernel without static LDS: checked here, once per device, before the first launch (a kernel
// that fails the check is never launched and the call returns VLUT_ERR_DEVICE).
bool allow_dynamic_lds(const void* kfn, int bytes, std::atomic<unsigned>& done_mask, bool needs_lds_base0 = true) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const unsigned bit = (dev >= 0 && dev < 32) ? (1u << dev) : 0u;
    if (bit && (done_mask.load(std::memory_order_relaxed) & bit)) return true;
    hipFuncAttributes attr;
    if (needs_lds_base0 && (hipFuncGetAttributes(&attr, kfn) != hipSuccess || attr.sharedSizeBytes != 0)) return false;
    if (hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    done_mask.fetch_or(bit, std::memory_order_relaxed);
    return true;
}

struct Plan {
    int Jlog, R, S;
    int BW;      // build waves of the 16-wave workgroup (4, 2 or 1); the other 16 - BW waves look up
};

thread_local Plan t_forced = {-1, 0, 0, 0};

const int kSupportedR[] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16};

bool r_supported(int R) {
    for (int v : kSupportedR)
        if (v == R) return true;
    return false;
}

bool shape_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && N >= 1 && K >= 4 && (K % 4) == 0 && M < kMaxDim && K < kMaxDim && N < kMaxDim;
}

struct Derived {
    int G, KCn, RGtotal, n_tile, tiles_n, tiles_m, RGW, stages_total, stages_per_split, total, per_xcd;
    bool need32;
};

Derived derive(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    Derived d;
    d.G = (int)(K / 4);
    d.KCn = (d.G + 15) / 16;
    d.RGtotal = (int)((M + 3) / 4);
    int J = 1 << pl.Jlog;
    d.n_tile = 128 >> pl.Jlog;
    d.tiles_n = (int)((N + d.n_tile - 1) / d.n_tile);
    int cap = (kWaves - pl.BW) * pl.R;                // row groups a workgroup can hold
    d.tiles_m = (d.RGtotal + cap - 1) / cap;
    d.RGW = (d.RGtotal + d.tiles_m - 1) / d.tiles_m;  // balanced rows per workgroup
    d.stages_total = (d.G + 4 * J - 1) / (4 * J);
    d.stages_per_split = (d.stages_total + pl.S - 1) / pl.S;
    d.total = d.tiles_m * d.tiles_n * pl.S;
    d.per_xcd = (d.total + 7) / 8;
    d.need32 = d.stages_per_split * 4 > kBlockLookups;
    return d;
}

// Cost model in nanoseconds, fitted to K-scans and in-kernel timestamps on this chip.  A stage (4 slots = 64
// k-groups at 16 sub-tables per table row) costs a fixed part (the table build and its LDS writes, which share the LDS
// pipe with the table reads) plus a part per row group of the slowest lookup wave (two table reads, two address
// permutes and four three-operand adds per slot pair); with two build waves the fixed part is smaller and every
// workgroup holds 7/6 of the rows, but the build itself takes ~1.37 us per stage, which only R >= 7 hides.  Per tile,
// outside the K loop: the cross-lane reduction and the stores of every row group (bound by the SIMD that holds the
// most lookup waves: four of 14, three of 12) and the hand-over to the next tile; once per workgroup: the argument
// fetch, the first activations and the first table.
double plan_cost(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    Derived d = derive(pl, M, K, N);
    const int lookup_waves = kWaves - pl.BW;
    const double rw = (double)((d.RGW + lookup_waves - 1) / lookup_waves);   // row groups of the slowest lookup wave
    double stage, outside;
    if (pl.BW == 4) {
        stage = 867.0 + 90.0 * rw;
        outside = 600.0 + 190.0 * rw;
    } else {
        stage = 745.0 + 106.0 * rw;
        if (stage < 1370.0) stage = 1370.0;
        outside = 600.0 + 250.0 * rw;
    }
    double wg = d.stages_per_split * stage * (d.need32 ? 1.05 : 1.0) + outside;
    double rounds = (double)((d.total + 255) / 256);          // tiles of the busiest workgroup
    double t = 2000.0 + 2100.0 + rounds * wg;
    if (pl.S > 1) t += 2400.0 + 290.0 * pl.S + (double)pl.S * (double)M * (double)N * 8.0 / (256.0 * 16.0 * 2.1);   // second kernel
    // weight bytes pulled from L2 by all token tiles (256 CUs x ~24 B/clk)
    double traffic = (double)d.tiles_n * (double)d.RGtotal * d.KCn * 64.0 / (256.0 * 24.0 * 2.1);
    return t > traffic ? t : traffic;
}

bool plan_valid(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    if (pl.Jlog < 0 || pl.Jlog > 4 || !r_supported(pl.R) || pl.S < 1 || pl.S > 16) return false;
    if (pl.BW != 4 && pl.BW != 2 && pl.BW != 1) return false;
    Derived d = derive(pl, M, K, N);
    if (d.need32 && pl.R > 6) return false;      // register budget of the INT32 variant
    if (pl.S > d.stages_total) return false;
    return true;
}

// A plan with R == 0 means: the override of vlut_set_plan fits this shape with no value of the free parameters
// (callers report VLUT_ERR_UNSUPPORTED).  Without an override there is always a valid plan (R = 1, S = 1).
const int kBuildWaveChoices[] = {4, 2};
Plan search_plan(int64_t M, int64_t K, int64_t N, int max_S = 16, bool four_build_waves_only = false) {
    Plan best = {0, 0, 0, 0};
    double best_cost = 1e300;
    const int Ss[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int Jlog = 0; Jlog <= 4; ++Jlog)
        for (int R : kSupportedR)
            for (int S : Ss) {
                if (S > max_S) continue;
                for (int BW : kBuildWaveChoices) {
                    if (four_build_waves_only && BW != 4) continue;
                    Plan pl = {t_forced.Jlog >= 0 ? t_forced.Jlog : Jlog, t_forced.R > 0 ? t_forced.R : R,
                               t_forced.S > 0 ? t_forced.S : S, t_forced.BW > 0 ? t_forced.BW : BW};
                    if (!plan_valid(pl, M, K, N)) continue;
                    double c = plan_cost(pl, M, K, N);
                    if (c < best_cost) { best_cost = c; best = pl; }
                }
            }
    return best;
}

// Fused quantisation needs 8-token tiles (16 sub-tables per row) and the codes of the workgroup's K range in LDS.
bool fused_plan_valid(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    if (pl.Jlog != 4 || pl.R > kFusedMaxR || !plan_valid(pl, M, K, N)) return false;
    return derive(pl, M, K, N).stages_per_split <= kFusedMaxStages;
}

bool search_fused_plan(int64_t M, int64_t K, int64_t N, Plan* out) {
    if ((t_forced.Jlog >= 0 && t_forced.Jlog != 4) || (t_forced.BW != 0 && t_forced.BW != 4)) return false;
    bool found = false;
    double best_cost = 1e300;
    const int Ss[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int R : kSupportedR)
        for (int S : Ss) {
            Plan pl = {4, t_forced.R > 0 ? t_forced.R : R, t_forced.S > 0 ? t_forced.S : S, 4};
            if (!fused_plan_valid(pl, M, K, N)) continue;
            double c = plan_cost(pl, M, K, N);
            if (c < best_cost) { best_cost = c; *out = pl; found = true; }
        }
    return found;
}

// The search above costs microseconds of host time; a launch-bound caller repeats a handful of shapes, so the
// last few answers are kept per thread (invalidated by vlut_set_plan).
struct PlanCacheEntry {
    int64_t M, K, N;
    Plan plan;
};
thread_local PlanCacheEntry t_cache[8];
thread_local int t_cache_used = 0, t_cache_next = 0;

Plan choose_plan(int64_t M, int64_t K, int64_t N) {
    for (int i = 0; i < t_cache_used; ++i)
        if (t_cache[i].M == M && t_cache[i].K == K && t_cache[i].N == N) return t_cache[i].plan;
    Plan pl = search_plan(M, K, N);
    t_cache[t_cache_next] = {M, K, N, pl};
    t_cache_next = (t_cache_next + 1) % 8;
    if (t_cache_used < 8) ++t_cache_used;
    return pl;
}

struct FusedCacheEntry {
    int64_t M, K, N;
    Plan plan;
    bool found;
};
thread_local FusedCacheEntry t_fcache[8];
thread_local int t_fcache_used = 0, t_fcache_next = 0;

bool choose_fused_plan(int64_t M, int64_t K, int64_t N, Plan* out) {
    for (int i = 0; i < t_fcache_used; ++i)
        if (t_fcache[i].M == M && t_fcache[i].K == K && t_fcache[i].N == N) {
            *out = t_fcache[i].plan;
            return t_fcache[i].found;
        }
    Plan pl = {4, 1, 1, 4};
    const bool found = search_fused_plan(M, K, N, &pl);
    t_fcache[t_fcache_next] = {M, K, N, pl, found};
    t_fcache_next = (t_fcache_next + 1) % 8;
    if (t_fcache_used < 8) ++t_fcache_used;
    *out = pl;
    return found;
}

// Compute units of the current device (cached per device; 0 if the query fails).
int compute_units() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 0;
    cached[dev].store(v, std::memory_order_relaxed);
    return v;
}

// The lookup kernel's workgroups are persistent: at most one per compute unit (a workgroup needs more than half of a
// unit's LDS), spread evenly over the 8 XCDs; each walks through its share of the tile list.
template <int R, bool NEED32, int MODE, int BW>
int launch_lookup_t(const LookupParams& p, hipStream_t stream) {
    const int cus = compute_units();
    if (cus < 8) return VLUT_ERR_DEVICE;
    const int grid = 8 * std::min(p.per_xcd, cus / 8);
    auto kfn = lookup_kernel<R, NEED32, MODE, BW>;
    constexpr int max_lds = MODE == kFusedQuant ? kFusedMaxLds : kLdsBytes;
    const int lds = MODE == kFusedQuant ? kFusedAqBase + p.stages_per_split * kFusedStageBytes : kLdsBytes;
    if (lds > max_lds) return VLUT_ERR_UNSUPPORTED;
    static std::atomic<unsigned> attr_done{0};   // one bit per device: the attribute belongs to the device's copy
    if (!allow_dynamic_lds((const void*)kfn, max_lds, attr_done)) return VLUT_ERR_DEVICE;
    LookupParams q = p;
    if (q.S > 1 || q.partial) q.out_vec = ((uintptr_t)q.ws % 16 == 0) && (q.M % 4 == 0);
    else q.out_vec = !q.y || (((uintptr_t)q.y % 16 == 0) && (q.ldy % 4 == 0));
    q.magic_S = q.S > 1 ? (unsigned)((1ull << 32) / (unsigned)q.S) : 0xffffffffu;
    q.magic_tiles_n = q.tiles_n > 1 ? (unsigned)((1ull << 32) / (unsigned)q.tiles_n) : 0xffffffffu;
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(kThreads), lds, stream, q);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

// Which instances of the lookup kernel are compiled: the streamed kernels for every supported R (the INT32-widening
// and the quantising variants hold more state per wave and stop earlier), the variant that reads a materialised
// table for a few small R only (the launcher maps R down).  VLUT_ONLY_R (a build-time macro for experiments)
// restricts the streamed instances to one R.
constexpr bool lookup_instance_built(int R, bool need32, int mode) {
#ifdef VLUT_ONLY_R
    if (mode != kFromGlobal && R != (VLUT_ONLY_R)) return false;
#endif
    if (mode == kFromGlobal) return R == 1 || R == 2 || R == 4;
    if (need32) return R <= 6;
    if (mode == kFusedQuant) return R <= kFusedMaxR;
    return R <= 16;
}

constexpr bool lookup_bw_built(int BW, int mode) { return BW == 4 || (BW == 2 && mode == kFast); }

template <bool NEED32, int MODE, int BW, int R = 1>
int launch_lookup_by_r(int r, const LookupParams& p, hipStream_t stream) {
    if constexpr (R > 16) {
        return VLUT_ERR_UNSUPPORTED;
    } else {
        if constexpr (lookup_instance_built(R, NEED32, MODE)) {
            if (r == R) return launch_lookup_t<R, NEED32, MODE, BW>(p, stream);
        }
        return launch_lookup_by_r<NEED32, MODE, BW, R + 1>(r, p, stream);
    }
}

template <bool NEED32>
int launch_lookup_r(int R, int BW, int mode, const LookupParams& p, hipStream_t stream) {
    if (mode == kFusedQuant && BW == 4) return launch_lookup_by_r<NEED32, kFusedQuant, 4>(R, p, stream);
    if (mode == kFast && BW == 4) return launch_lookup_by_r<NEED32, kFast, 4>(R, p, stream);
    if (mode == kFast && BW == 2) return launch_lookup_by_r<NEED32, kFast, 2>(R, p, stream);
    if (mode == kFromGlobal && BW == 4) return launch_lookup_by_r<NEED32, kFromGlobal, 4>(R, p, stream);
    return VLUT_ERR_UNSUPPORTED;
}

// Second kernel of a split-K (or mixed-packing) launch: four rows per thread when everything is aligned for it.
int launch_splitk_reduce(const int32_t* ws, int S, int64_t M, int64_t N, float w_scale, const float* w_rows,
                         const float* a_scale, float* y, int64_t ldy, int32_t* acc, hipStream_t s) {
    const bool vec = (M % 4 == 0) && ((uintptr_t)ws % 16 == 0) && (!y || ((uintptr_t)y % 16 == 0 && ldy % 4 == 0)) &&
                     (!w_rows || (uintptr_t)w_rows % 16 == 0);
    const size_t total = (size_t)(vec ? M / 4 : M) * (size_t)N;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (vec) hipLaunchKernelGGL(splitk_reduce_kernel<4>, grid, dim3(256), 0, s, ws, S, (int)M, (int)N, w_scale, w_rows,
                                a_scale, y, ldy, acc);
    else hipLaunchKernelGGL(splitk_reduce_kernel<1>, grid, dim3(256), 0, s, ws, S, (int)M, (int)N, w_scale, w_rows,
                            a_scale, y, ldy, acc);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

int check_mpgemm_args(const uint8_t* packed, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                      int64_t N, float* y, int64_t ldy, int32_t* acc) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !a_q || !a_scale) return VLUT_ERR_NULL;
    if (!y && !acc) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    return VLUT_OK;
}

// ---- few-token kernel: one copy of the row tiles per token pair.  Measured (K = 2560..6912, 40..250 workgroups):
//      the time of a launch depends on the rows per workgroup, hardly on the number of workgroups while they all
//      fit the device at once (16 rows with four lanes per row were never the best), against 12-16 us for quantiser
//      + general kernel + split-K sum at 3..32 tokens.  So: the fewest rows (from 32) whose grid is one round of
//      workgroups, and narrow_applies weighs that against the general path.
constexpr int kNarrowMaxN = 32;
struct NarrowPlan {
    int parts, rr, rows, gridx, chunks, pairs, gx8, grid;
};

NarrowPlan narrow_plan(int64_t M, int64_t K, int64_t N) {
    NarrowPlan np;
    np.pairs = (int)((N + 1) / 2);
    for (int rows = 32; rows <= 256; rows *= 2) {
        np.rows = rows;
        np.gridx = (int)((M + rows - 1) / rows);
        np.gx8 = np.pairs > 1 ? (np.gridx + 7) / 8 * 8 : np.gridx;
        const int64_t grid = (int64_t)np.gx8 * (np.pairs - 1) + np.gridx;
        np.grid = (int)(grid < INT32_MAX ? grid : INT32_MAX);
        if (grid <= 256) break;
    }
    np.parts = np.rows == 32 ? 2 : 1;
    np.rr = np.rows <= 64 ? 1 : np.rows / 64;
    np.chunks = (int)((K / 4 + kNarrowChunk - 1) / kNarrowChunk);
    return np;
}

// One or two tokens always take this kernel; more tokens while its workgroups fit the device at once and a cost
// estimate fitted to measurements at N <= 32 (2B-model shapes) favours it by 10 %.  In us, with c = K / 1024:
//   this kernel   4.6 from fp32 activations (3.6 from INT8 ones) + c x {0.9, 1.35, 2.0, 3.4} for 32, 64, 128, 256 rows
//                 per workgroup;
//   general path  5.8 + 0.94 c + 0.41 x M N / 10^4 for lookup kernel + split-K sum, + 3.5 for the quantiser from fp32.
bool narrow_applies(int64_t M, int64_t K, int64_t N, const void* lut, bool from_f32) {
    if (N > kNarrowMaxN || lut != nullptr || t_forced.Jlog >= 0 || t_forced.R != 0 || t_forced.S != 0 || t_forced.BW != 0) return false;
    if (N <= 2) return true;
    const NarrowPlan np = narrow_plan(M, K, N);
    if (np.grid > 256) return false;
    const double c = (double)K / 1024.0;
    const double per_chunk = np.rows <= 32 ? 0.9 : (np.rows <= 64 ? 1.35 : (np.rows <= 128 ? 2.0 : 3.4));
    const double narrow_us = (from_f32 ? 4.6 : 3.6) + c * per_chunk;
    const double general_us = 5.8 + 0.94 * c + 0.41 * (double)M * (double)N / 1e4 + (from_f32 ? 3.5 : 0.0);
    return narrow_us * 1.1 < general_us;
}

template <int NTOK, int PARTS, int RR, bool FUSED>
int launch_narrow_t(const NarrowParams& p, int grid, hipStream_t stream) {
    auto kfn = narrow_kernel<NTOK, PARTS, RR, FUSED>;
    constexpr int max_lds = FUSED ? 160 * 1024 : narrow_tab_bytes(NTOK);
    const int lds = FUSED ? narrow_fused_lds_bytes(NTOK, p.chunks) : narrow_tab_bytes(NTOK);
    if (lds > max_lds) return VLUT_ERR_UNSUPPORTED;
    static std::atomic<unsigned> attr_done{0};   // one bit per device: the attribute belongs to the device's copy
    if (!allow_dynamic_lds((const void*)kfn, max_lds, attr_done)) return VLUT_ERR_DEVICE;
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(kThreads), lds, stream, p);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

template <int NTOK, bool FUSED>
int launch_narrow_n(const NarrowPlan& np, const NarrowParams& p, hipStream_t stream) {
    if (np.parts == 2) return launch_narrow_t<NTOK, 2, 1, FUSED>(p, np.grid, stream);
    if (np.rr == 1) return launch_narrow_t<NTOK, 1, 1, FUSED>(p, np.grid, stream);
    if (np.rr == 2) return launch_narrow_t<NTOK, 1, 2, FUSED>(p, np.grid, stream);
    return launch_narrow_t<NTOK, 1, 4, FUSED>(p, np.grid, stream);
}

template <bool FUSED>
int launch_narrow(const NarrowPlan& np, const NarrowParams& p, hipStream_t stream) {
    NarrowParams q = p;
    q.gridx = np.gridx;
    q.gx8 = np.gx8;
    q.chunks = np.chunks;
    return q.N == 1 ? launch_narrow_n<1, FUSED>(np, q, stream) : launch_narrow_n<2, FUSED>(np, q, stream);
}

std::mutex g_pack_mutex;

// ---- vlut_mpgemm_f32: which kernels run and how the caller's workspace is divided
enum { kF32Narrow = 0, kF32Fused = 1, kF32TwoLaunches = 2 };
struct F32Layout {
    int kind;
    Plan plan;                                   // kF32Fused
    size_t off_scale, off_amax, off_aq, off_ws, total;     // byte offsets into the workspace
};

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// Inputs from which the two-kernel quantiser (absmax per token, then chunks of 8 tokens per K range) is the fastest
// form (measured: 14.6 against 21.2 us at N = 512, K = 14336; a second launch costs more than it saves below about
// four million values); it needs N floats of scratch, which only vlut_mpgemm_f32 has (its workspace).
bool quantize_two_kernels(int64_t N, int64_t K) { return N * K >= ((int64_t)1 << 22) && N >= 64; }

F32Layout f32_layout(int64_t M, int64_t K, int64_t N) {
    F32Layout L;
    std::memset(&L, 0, sizeof(L));
    const size_t scale_bytes = round256((size_t)N * sizeof(float));
    if (narrow_applies(M, K, N, nullptr, true) && narrow_plan(M, K, N).chunks <= narrow_fused_max_chunks(N == 1 ? 1 : 2)) {
        L.kind = kF32Narrow;
        return L;
    }
    // More than two tokens: measured, quantising inside the lookup kernel loses against a kernel of its own ahead of
    // it (every workgroup reads the whole rows of its 8 tokens and 16 row tiles repeat the work: +5.6 us on the
    // lookup kernel at M = 6912, K = 2560, N = 128, against 3.2 us + the gap between two kernels).  The fused form
    // is therefore only taken when a launch plan is forced (an override selects the kernel too).
    const bool forced = t_forced.Jlog >= 0 || t_forced.R > 0 || t_forced.S > 0 || t_forced.BW > 0;
    const bool fused = forced && choose_fused_plan(M, K, N, &L.plan);
    if (fused) {
        L.kind = kF32Fused;
        if (L.plan.S > 1) {                      // the second kernel reads the scales from memory
            L.off_ws = scale_bytes;
            L.total = L.off_ws + (size_t)L.plan.S * (size_t)M * (size_t)N * sizeof(int32_t);
        }
        return L;
    }
    L.kind = kF32TwoLaunches;                    // quantise into the workspace, then the ordinary path
    L.off_amax = scale_bytes;                    // per-token absmax between the two kernels of the quantiser
    L.off_aq = L.off_amax + (quantize_two_kernels(N, K) ? scale_bytes : 0);
    L.off_ws = L.off_aq + round256((size_t)((N + 7) / 8) * (size_t)K * 8);
    const bool narrow = narrow_applies(M, K, N, nullptr, false);
    const Plan pl = narrow ? Plan{4, 1, 1, 4} : choose_plan(M, K, N);
    L.plan = pl;
    L.total = L.off_ws + (pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0);
    return L;
}

// ---- 1.60-bit (g = 5) host side
struct Plan5 {
    int R, S;
};
thread_local Plan5 t_forced5 = {0, 0};
constexpr int kSupportedR5[] = {1, 2, 4, 6, 9, 12, 14};

bool shape5_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && N >= 1 && K >= 5 && (K % 5) == 0 && M < kMaxDim && K < kMaxDim && N < kMaxDim;
}

struct Derived5 {
    int G, KCn, RGtotal, tiles_n, tiles_m, RGW, dstages_total, dstages_per_split, total, per_xcd;
    bool need32;
};

Derived5 derive5(const Plan5& pl, int64_t M, int64_t K, int64_t N) {
    Derived5 d;
    d.G = (int)(K / 5);
    d.KCn = (d.G + 15) / 16;
    d.RGtotal = (int)((M + 3) / 4);
    d.tiles_n = (int)((N + 7) / 8);
    int cap = kLookupWaves5 * pl.R;
    d.tiles_m = (d.RGtotal + cap - 1) / cap;
    d.RGW = (d.RGtotal + d.tiles_m - 1) / d.tiles_m;
    d.dstages_total = (d.G + 63) / 64;
    d.dstages_per_split = (d.dstages_total + pl.S - 1) / pl.S;
    d.total = d.tiles_m * d.tiles_n * pl.S;
    d.per_xcd = (d.total + 7) / 8;
    d.need32 = d.dstages_per_split * 4 > kBlockLookups5;
    return d;
}

bool plan5_valid(const Plan5& pl, int64_t M, int64_t K, int64_t N) {
    bool ok = false;
    for (int v : kSupportedR5) ok = ok || v == pl.R;
    if (!ok || pl.S < 1 || pl.S > 16) return false;
    Derived5 d = derive5(pl, M, K, N);
    if (d.need32 && pl.R > 6) return false;
    return pl.S <= d.dstages_total;
}

// R == 0 in the result: the override of vlut_set_plan_g5 fits this shape with no value of the free parameter
// (plan5_valid is then false and the callers report VLUT_ERR_UNSUPPORTED).
Plan5 choose_plan5(int64_t M, int64_t K, int64_t N) {
    Plan5 best = {0, 0};
    double best_cost = 1e300;
    const int Ss[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int R : kSupportedR5)
        for (int S : Ss) {
            Plan5 pl = {t_forced5.R > 0 ? t_forced5.R : R, t_forced5.S > 0 ? t_forced5.S : S};
            if (!plan5_valid(pl, M, K, N)) continue;
            Derived5 d = derive5(pl, M, K, N);
            double rw = (double)((d.RGW + kLookupWaves5 - 1) / kLookupWaves5);
            // a dword stage = four half-stages; each writes a 62 KB slot and reads it rw times per lookup wave
            double wg = d.dstages_per_split * 4.0 * (1900.0 + 75.0 * rw) + 5900.0 + 840.0 * rw;
            double t = (double)((d.total + 255) / 256) * wg;
            if (pl.S > 1) t += 5000.0 + 600.0 * pl.S;
            if (t < best_cost) { best_cost = t; best = pl; }
        }
    return best;
}

template <int R, bool NEED32>
int launch_lookup5_t(const Lookup5Params& p, int grid, hipStream_t stream) {
    auto kfn = lookup5_kernel<R, NEED32>;
    static std::atomic<unsigned> attr_done{0};   // one bit per device: the attribute belongs to the device's copy
    if (!allow_dynamic_lds((const void*)kfn, kLds5Bytes, attr_done)) return VLUT_ERR_DEVICE;
    Lookup5Params q = p;
    if (q.S > 1 || q.partial) q.out_vec = ((uintptr_t)q.ws % 16 == 0) && (q.M % 4 == 0);
    else q.out_vec = !q.y || (((uintptr_t)q.y % 16 == 0) && (q.ldy % 4 == 0));
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(kThreads), kLds5Bytes, stream, q);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

template <bool NEED32>
int launch_lookup5_r(int R, const Lookup5Params& p, int grid, hipStream_t stream);

constexpr bool lookup5_instance_built(int R, bool need32) {
    for (int v : kSupportedR5)
        if (v == R) return !need32 || R <= 6;
    return false;
}

template <bool NEED32, int R = 1>
int launch_lookup5_by_r(int r, const Lookup5Params& p, int grid, hipStream_t stream) {
    if constexpr (R > 14) {
        return VLUT_ERR_UNSUPPORTED;
    } else {
        if constexpr (lookup5_instance_built(R, NEED32)) {
            if (r == R) return launch_lookup5_t<R, NEED32>(p, grid, stream);
        }
        return launch_lookup5_by_r<NEED32, R + 1>(r, p, grid, stream);
    }
}

template <bool NEED32>
int launch_lookup5_r(int R, const Lookup5Params& p, int grid, hipStream_t stream) {
    return launch_lookup5_by_r<NEED32>(R, p, grid, stream);
}

// ---- comparison path: tokens per workgroup from N, K split so that few tiles still give every CU a few workgroups
struct MfmaPlan {
    int BN, tiles_m, tiles_n, S, steps_per_split, grid;
};

MfmaPlan mfma_plan(int64_t M, int64_t K, int64_t N) {
    MfmaPlan mp;
    mp.BN = N > 64 ? 128 : (N > 32 ? 64 : (N > 16 ? 32 : 16));
    mp.tiles_m = (int)((M + kMfRows - 1) / kMfRows);
    // the kernel hides latency with resident waves only: narrower token tiles while the wide ones give a CU fewer
    // than about three workgroups
    if (mp.BN == 128 && (int64_t)mp.tiles_m * ((N + 127) / 128) < 768) mp.BN = 64;
    mp.tiles_n = (int)((N + mp.BN - 1) / mp.BN);
    const int steps = (int)((K / 4 + 15) / 16);
    const int64_t tiles = (int64_t)mp.tiles_m * mp.tiles_n;
    int S = 1;
    if (tiles < 512) {
        S = (int)((768 + tiles - 1) / tiles);                // about three workgroups per CU
        if (S > 16) S = 16;
        if (S > steps / 4) S = steps / 4 > 0 ? steps / 4 : 1;  // at least four K steps per split
    }
    mp.steps_per_split = (steps + S - 1) / S;
    mp.S = (steps + mp.steps_per_split - 1) / mp.steps_per_split;
    mp.grid = (int)(tiles * mp.S);
    return mp;
}

}  // namespace

extern "C" {

const char* vlut_status_string(int status) {
    switch (status) {
    case VLUT_OK: return "VLUT_OK";
    case VLUT_ERR_NULL: return "VLUT_ERR_NULL: a required pointer is NULL";
    case VLUT_ERR_SHAPE: return "VLUT_ERR_SHAPE: shape or leading dimension out of range";
    case VLUT_ERR_SMALL_BUFFER: return "VLUT_ERR_SMALL_BUFFER: buffer smaller than required";
    case VLUT_ERR_VALUE: return "VLUT_ERR_VALUE: weight outside {-1,0,+1}";
    case VLUT_ERR_DEVICE: return "VLUT_ERR_DEVICE: HIP call or kernel launch failed";
    case VLUT_ERR_UNSUPPORTED: return "VLUT_ERR_UNSUPPORTED: request not supported by this build";
    default: return "VLUT_ERR_UNKNOWN";
    }
}

int vlut_version(void) { return 100; }

size_t vlut_packed_weight_bytes(int64_t M, int64_t K) {
    if (!shape_ok(M, K, 1)) return 0;
    return (size_t)((M + 3) / 4) * (size_t)((K / 4 + 15) / 16) * 64;
}

size_t vlut_packed_offset(int64_t M, int64_t K, int64_t m, int64_t kg) {
    if (!shape_ok(M, K, 1) || m < 0 || m >= M || kg < 0 || kg >= K / 4) return (size_t)-1;
    size_t KCn = (size_t)((K / 4 + 15) / 16);
    return (((size_t)(m / 4) * KCn + (size_t)(kg / 16)) * 64) + (size_t)(m % 4) * 16 + (size_t)(kg % 16);
}

size_t vlut_act_bytes(int64_t K, int64_t N) {
    if (!shape_ok(1, K, N)) return 0;
    return (size_t)((N + 7) / 8) * (size_t)K * 8;
}

size_t vlut_lut_bytes(int64_t K, int64_t N) {
    if (!shape_ok(1, K, N)) return 0;
    return (size_t)(K / 4) * kRows * (size_t)N * sizeof(int16_t);
}

size_t vlut_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    // Where the few-token kernel serves the streamed path (no workspace), the materialised-table variant runs a
    // plan without split-K, so this one size serves both variants.
    if (narrow_applies(M, K, N, nullptr, false)) return 0;
    const Plan pl = choose_plan(M, K, N);
    return pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
}

int vlut_set_plan(int J, int R, int waves, int split_k) {
    int Jlog = -1;
    if (J != 0) {
        for (int e = 0; e <= 4; ++e)
            if ((1 << e) == J) Jlog = e;
        if (Jlog < 0) return VLUT_ERR_UNSUPPORTED;
    }
    if (R != 0 && !r_supported(R)) return VLUT_ERR_UNSUPPORTED;
    if (waves != 0 && waves != kWaves && waves != 12 && waves != 14) return VLUT_ERR_UNSUPPORTED;
    if (split_k < 0 || split_k > 16) return VLUT_ERR_UNSUPPORTED;
    t_forced = {Jlog, R, split_k, (waves == 12 || waves == 14) ? kWaves - waves : 0};
    t_cache_used = 0;
    t_cache_next = 0;
    t_fcache_used = 0;
    t_fcache_next = 0;
    return VLUT_OK;
}

int vlut_query_plan(int64_t M, int64_t K, int64_t N, int* out4) {
    if (!out4) return VLUT_ERR_NULL;
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (narrow_applies(M, K, N, nullptr, false)) {   // the few-token kernel: J reported as 0, R = rows per workgroup
        const NarrowPlan np = narrow_plan(M, K, N);
        out4[0] = 0; out4[1] = np.rows; out4[2] = 1; out4[3] = np.gridx * np.pairs;
        return VLUT_OK;
    }
    Plan pl = choose_plan(M, K, N);
    if (pl.R == 0) return VLUT_ERR_UNSUPPORTED;          // the override does not fit this shape
    Derived d = derive(pl, M, K, N);
    out4[0] = 1 << pl.Jlog;
    out4[1] = pl.R;
    out4[2] = pl.S;
    out4[3] = d.total;
    return VLUT_OK;
}

int vlut_query_lookup_waves(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (narrow_applies(M, K, N, nullptr, false)) return 0;
    const Plan pl = choose_plan(M, K, N);
    if (pl.R == 0) return VLUT_ERR_UNSUPPORTED;
    return kWaves - pl.BW;
}

int vlut_pack_weights(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                      void* stream) {
    if (!shape_ok(M, K, 1)) return VLUT_ERR_SHAPE;
    if (!w_ternary || !packed) return VLUT_ERR_NULL;
    size_t need = vlut_packed_weight_bytes(M, K);
    if (packed_bytes < need) return VLUT_ERR_SMALL_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_pack_mutex);
    int zero = 0;
    if (hipMemcpyToSymbolAsync(HIP_SYMBOL(g_pack_error), &zero, sizeof(int), 0, hipMemcpyHostToDevice, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    int G = (int)(K / 4), KCn = (G + 15) / 16, RGtotal = (int)((M + 3) / 4);
    size_t blocks = (need + 255) / 256;
    hipLaunchKernelGGL(pack_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, s, w_ternary, (int)M, K, G, KCn, RGtotal,
                       packed);
    if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    int err = 0;
    if (hipMemcpyFromSymbolAsync(&err, HIP_SYMBOL(g_pack_error), sizeof(int), 0, hipMemcpyDeviceToHost, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return VLUT_ERR_DEVICE;
    return err ? VLUT_ERR_VALUE : VLUT_OK;
}

#ifndef VLUT_QUANT_PER_TOKEN
// measured: the per-token kernel is the faster one except for more than ~2M values in short rows, where its
// single-byte stores cost more than the chunk kernel's serial reads
#define VLUT_QUANT_PER_TOKEN(N, K) (!((N) * (K) >= 2000000 && (K) <= 4096))
#endif
static int quantize_impl(const float* x, int64_t N, int64_t K, int64_t ldx, int8_t* a_q, float* a_scale,
                         float* amax_scratch_or_null, void* stream) {
    if (!shape_ok(1, K, N)) return VLUT_ERR_SHAPE;
    if (ldx < K) return VLUT_ERR_SHAPE;
    if (!x || !a_q || !a_scale) return VLUT_ERR_NULL;
    if (((uintptr_t)a_q) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    const unsigned chunks = (unsigned)((N + 7) / 8);
    const bool vec = (((uintptr_t)x) % 16 == 0) && (ldx % 4 == 0);
    if (amax_scratch_or_null && quantize_two_kernels(N, K)) {
        if (vec) hipLaunchKernelGGL(absmax_token_kernel<true>, dim3((unsigned)N), dim3(kTokThreads), 0, s, x, (int)N, (int)K, ldx,
                                    amax_scratch_or_null);
        else hipLaunchKernelGGL(absmax_token_kernel<false>, dim3((unsigned)N), dim3(kTokThreads), 0, s, x, (int)N, (int)K, ldx,
                                amax_scratch_or_null);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
        // K ranges per chunk: enough workgroups for about three per CU, each at least one pass of 256 quads
        const int nquad = (int)(K / 4);
        int ranges = (int)((768 + chunks - 1) / chunks);
        const int max_ranges = (nquad + kTokThreads - 1) / kTokThreads;
        if (ranges > max_ranges) ranges = max_ranges;
        if (ranges < 1) ranges = 1;
        int quads_per_block = (nquad + ranges - 1) / ranges;
        quads_per_block = (quads_per_block + kTokThreads - 1) / kTokThreads * kTokThreads;
        ranges = (nquad + quads_per_block - 1) / quads_per_block;
        const dim3 grid(chunks, (unsigned)ranges);
        if (vec) hipLaunchKernelGGL(quantize_chunk_kernel<true>, grid, dim3(kTokThreads), 0, s, x, (int)N, (int)K, ldx,
                                    (const float*)amax_scratch_or_null, a_q, a_scale, quads_per_block);
        else hipLaunchKernelGGL(quantize_chunk_kernel<false>, grid, dim3(kTokThreads), 0, s, x, (int)N, (int)K, ldx,
                                (const float*)amax_scratch_or_null, a_q, a_scale, quads_per_block);
        return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
    }
    const size_t lds = (size_t)K * 8;
    const int nquad_per_thread = (int)((K / 4 + 127) / 128);
    auto launch = [&](auto kfn) -> int {
        if (lds > 160 * 1024 - 1024) return VLUT_ERR_UNSUPPORTED;   // the chunk's [K][8] block is staged in LDS
        static std::atomic<unsigned> attr_done{0};   // per kernel instance (generic lambda), one bit per device
        if (lds > 48 * 1024 && !allow_dynamic_lds((const void*)kfn, 160 * 1024 - 1024, attr_done, false))
            return VLUT_ERR_DEVICE;
        hipLaunchKernelGGL(kfn, dim3(chunks), dim3(kQuantThreads), lds, s, x, (int)N, (int)K, ldx, a_q, a_scale);
        return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
    };
    // One workgroup per token (every CU reads one row once) unless the byte stores would dominate
    if (VLUT_QUANT_PER_TOKEN(N, K)) {
        const unsigned blocks = ((chunks + 7) / 8) * 64;
        const int per_thread = (int)((K / 4 + kTokThreads - 1) / kTokThreads);
        auto launch_tok = [&](auto kfn) -> int {
            hipLaunchKernelGGL(kfn, dim3(blocks), dim3(kTokThreads), 0, s, x, (int)N, (int)K, ldx, a_q, a_scale, (int)chunks);
            return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
        };
        if (!vec) return launch_tok(quantize_token_kernel<0, false>);
        if (per_thread <= 4) return launch_tok(quantize_token_kernel<4, true>);
        if (per_thread <= 10) return launch_tok(quantize_token_kernel<10, true>);
        if (per_thread <= 16) return launch_tok(quantize_token_kernel<16, true>);
        return launch_tok(quantize_token_kernel<0, true>);
    }
    if (vec) {
        if (nquad_per_thread <= 5) return launch(quantize_kernel<5, true>);
        if (nquad_per_thread <= 8) return launch(quantize_kernel<8, true>);
        if (nquad_per_thread <= 16) return launch(quantize_kernel<16, true>);
        return launch(quantize_kernel<0, true>);
    }
    return launch(quantize_kernel<0, false>);
}

int vlut_quantize_act(const float* x, int64_t N, int64_t K, int64_t ldx, int8_t* a_q, float* a_scale,
                      void* stream) {
    return quantize_impl(x, N, K, ldx, a_q, a_scale, nullptr, stream);
}

int vlut_build_lut(const int8_t* a_q, int64_t K, int64_t N, int16_t* lut, size_t lut_bytes, void* stream) {
    if (!shape_ok(1, K, N)) return VLUT_ERR_SHAPE;
    if (!a_q || !lut) return VLUT_ERR_NULL;
    if (lut_bytes < vlut_lut_bytes(K, N)) return VLUT_ERR_SMALL_BUFFER;
    size_t total = (size_t)(K / 4) * (size_t)N;
    hipLaunchKernelGGL(build_lut_kernel<false>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       a_q, (int)(K / 4), (int)N, lut);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

int vlut_build_lut_token_outer(const int8_t* a_q, int64_t K, int64_t N, int16_t* lut, size_t lut_bytes, void* stream) {
    if (!shape_ok(1, K, N)) return VLUT_ERR_SHAPE;
    if (!a_q || !lut) return VLUT_ERR_NULL;
    if (lut_bytes < vlut_lut_bytes(K, N)) return VLUT_ERR_SMALL_BUFFER;
    size_t total = (size_t)(K / 4) * (size_t)N;
    hipLaunchKernelGGL(build_lut_kernel<true>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       a_q, (int)(K / 4), (int)N, lut);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

int vlut_mpgemm_token_outer(const uint8_t* packed, float w_scale, const float* a_scale, const int16_t* lut, int64_t M,
                            int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* stream) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !a_scale || !lut) return VLUT_ERR_NULL;
    if (!y && !acc_or_null) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    const int G = (int)(K / 4), KCn = (G + 15) / 16;
    const dim3 grid((unsigned)((M + 63) / 64), (unsigned)((N + 3) / 4));
    if (grid.y > 65535u) return VLUT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(token_outer_lookup_kernel, grid, dim3(256), 0, (hipStream_t)stream, packed, lut, (int)M, (int)N, G,
                       KCn, w_scale, a_scale, y, ldy, acc_or_null);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

static int mpgemm_impl(const uint8_t* packed, float w_scale, const float* w_rows, const int8_t* a_q, const float* a_scale,
                       const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                       int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    if (((uintptr_t)a_q) % 16 != 0) return VLUT_ERR_UNSUPPORTED;      // the [N/8][K][8] blocks are read 16 bytes at a time
    if (((uintptr_t)packed) % 16 != 0) return VLUT_ERR_UNSUPPORTED;   // packed tiles are read up to 16 bytes at a time
    if (narrow_applies(M, K, N, lut_or_null, false)) {   // a few tokens: the workgroups sweep all of K, no workspace
        const NarrowPlan np = narrow_plan(M, K, N);
        NarrowParams q;
        std::memset(&q, 0, sizeof(q));
        q.packed = packed; q.a_q = a_q; q.a_scale = a_scale; q.w_rows = w_rows; q.y = y; q.acc = acc_or_null;
        q.w_scale = w_scale; q.M = (int)M; q.K = (int)K; q.N = (int)N; q.G = (int)(K / 4);
        q.KCn = (int)((K / 4 + 15) / 16); q.RGtotal = (int)((M + 3) / 4); q.ldy = (int)ldy; q.chunks = np.chunks;
        return launch_narrow<false>(np, q, (hipStream_t)stream);
    }
    // A materialised table where the streamed path would take the few-token kernel (and vlut_workspace_bytes says
    // 0): a plan without split-K, so that no workspace is needed here either.
    Plan pl = (lut_or_null && narrow_applies(M, K, N, nullptr, false)) ? search_plan(M, K, N, 1) : choose_plan(M, K, N);
    if (lut_or_null && pl.R != 0 && pl.BW != 4) pl = search_plan(M, K, N, narrow_applies(M, K, N, nullptr, false) ? 1 : 16, true);
    if (pl.R == 0) return VLUT_ERR_UNSUPPORTED;          // the override of vlut_set_plan does not fit this shape
    const bool al = lut_or_null && (N % 8 == 0) && (((uintptr_t)lut_or_null) % 16 == 0);
    const int mode = lut_or_null ? kFromGlobal : kFast;
    if (mode != kFast) {   // the materialised-table variant is built for these R and four build waves only
        pl.R = pl.R >= 4 ? 4 : (pl.R >= 2 ? 2 : 1);
        pl.BW = 4;
    }
    Derived d = derive(pl, M, K, N);
    size_t ws_need = pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
    if (ws_need > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < ws_need) return VLUT_ERR_SMALL_BUFFER;
    }
    LookupParams p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.lut = lut_or_null;
    p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)workspace; p.w_scale = w_scale; p.w_rows = w_rows;
    p.M = (int)M; p.K = (int)K; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
    p.Jlog = pl.Jlog; p.S = pl.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
    p.stages_total = d.stages_total; p.stages_per_split = d.stages_per_split;
    p.total_tiles = d.total; p.per_xcd = d.per_xcd;
    p.aligned8 = al ? 1 : 0;
    p.Ka = (int)K;
    hipStream_t s = (hipStream_t)stream;
    rc = d.need32 ? launch_lookup_r<true>(pl.R, pl.BW, mode, p, s) : launch_lookup_r<false>(pl.R, pl.BW, mode, p, s);
    if (rc != VLUT_OK) return rc;
    if (pl.S > 1)
        return launch_splitk_reduce((const int32_t*)workspace, pl.S, M, N, w_scale, w_rows, a_scale, y, ldy, acc_or_null, s);
    return VLUT_OK;
}

int vlut_mpgemm(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale,
                const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    return mpgemm_impl(packed, w_scale, nullptr, a_q, a_scale, lut_or_null, M, K, N, y, ldy, acc_or_null, workspace,
                       workspace_bytes, stream);
}

size_t vlut_static_scratch_bytes(void) { return (size_t)VLUT_STATIC_SCRATCH_BYTES; }

int vlut_mpgemm_static(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                       int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    const size_t need = vlut_workspace_bytes(M, K, N);
    if (need > (size_t)VLUT_STATIC_SCRATCH_BYTES) return VLUT_ERR_UNSUPPORTED;   // partial sums beyond the built-in scratch
    void* ptr = nullptr;
    if (need > 0) {
        rc = static_scratch_ptr(&ptr);
        if (rc != VLUT_OK) return rc;
    }
    // Every partial-sum slot the second kernel reads is written by the first kernel of the same call, so nothing of
    // an earlier call's contents has to be cleared.
    return mpgemm_impl(packed, w_scale, nullptr, a_q, a_scale, nullptr, M, K, N, y, ldy, acc_or_null, ptr,
                       need > 0 ? (size_t)VLUT_STATIC_SCRATCH_BYTES : 0, stream);
}

int vlut_mpgemm_rows(const uint8_t* packed, const float* w_scale_rows, const int8_t* a_q, const float* a_scale,
                     const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                     int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    if (!w_scale_rows) return VLUT_ERR_NULL;
    return mpgemm_impl(packed, 1.0f, w_scale_rows, a_q, a_scale, lut_or_null, M, K, N, y, ldy, acc_or_null, workspace,
                       workspace_bytes, stream);
}

size_t vlut_workspace_bytes_f32(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    return f32_layout(M, K, N).total;
}

int vlut_query_plan_f32(int64_t M, int64_t K, int64_t N, int* out5) {
    if (!out5) return VLUT_ERR_NULL;
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    const F32Layout L = f32_layout(M, K, N);
    out5[4] = L.kind == kF32TwoLaunches ? 0 : 1;
    if (L.kind == kF32Fused) {
        const Derived d = derive(L.plan, M, K, N);
        out5[0] = 1 << L.plan.Jlog; out5[1] = L.plan.R; out5[2] = L.plan.S; out5[3] = d.total;
        return VLUT_OK;
    }
    if (L.kind == kF32Narrow) {                // reported as vlut_query_plan reports the few-token kernel
        const NarrowPlan np = narrow_plan(M, K, N);
        out5[0] = 0; out5[1] = np.rows; out5[2] = 1; out5[3] = np.gridx * np.pairs;
        return VLUT_OK;
    }
    return vlut_query_plan(M, K, N, out5);
}

int vlut_mpgemm_f32(const uint8_t* packed, float w_scale, const float* w_scale_rows_or_null, const float* x, int64_t ldx,
                    int64_t M, int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null,
                    float* a_scale_out_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !x) return VLUT_ERR_NULL;
    if (!y && !acc_or_null) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    if (ldx < K) return VLUT_ERR_SHAPE;
    if (((uintptr_t)packed) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    const F32Layout L = f32_layout(M, K, N);
    if (L.kind == kF32TwoLaunches && L.plan.R == 0) return VLUT_ERR_UNSUPPORTED;   // override does not fit the shape
    if (L.total > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < L.total) return VLUT_ERR_SMALL_BUFFER;
        if (((uintptr_t)workspace) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    }
    hipStream_t s = (hipStream_t)stream;
    const int x_vec = ((((uintptr_t)x) % 16 == 0) && (ldx % 4 == 0)) ? 1 : 0;
    const float* w_rows = w_scale_rows_or_null;
    const float w_one = w_rows ? 1.0f : w_scale;
    char* ws = (char*)workspace;

    if (L.kind == kF32Narrow) {
        const NarrowPlan np = narrow_plan(M, K, N);
        NarrowParams q;
        std::memset(&q, 0, sizeof(q));
        q.packed = packed; q.w_rows = w_rows; q.y = y; q.acc = acc_or_null; q.w_scale = w_one;
        q.M = (int)M; q.K = (int)K; q.N = (int)N; q.G = (int)(K / 4);
        q.KCn = (int)((K / 4 + 15) / 16); q.RGtotal = (int)((M + 3) / 4); q.ldy = (int)ldy; q.chunks = np.chunks;
        q.x = x; q.ldx = ldx; q.x_vec = x_vec; q.a_scale_out = a_scale_out_or_null;
        return launch_narrow<true>(np, q, s);
    }
    if (L.kind == kF32TwoLaunches) {
        float* scales = a_scale_out_or_null ? a_scale_out_or_null : (float*)(ws + L.off_scale);
        int8_t* a_q = (int8_t*)(ws + L.off_aq);
        int rc = quantize_impl(x, N, K, ldx, a_q, scales, quantize_two_kernels(N, K) ? (float*)(ws + L.off_amax) : nullptr,
                               stream);
        if (rc != VLUT_OK) return rc;
        return mpgemm_impl(packed, w_one, w_rows, a_q, scales, nullptr, M, K, N, y, ldy, acc_or_null, ws + L.off_ws,
                           L.total - L.off_ws, stream);
    }
    const Plan pl = L.plan;
    const Derived d = derive(pl, M, K, N);
    float* scales = a_scale_out_or_null;
    if (pl.S > 1 && !scales) scales = (float*)(ws + L.off_scale);
    LookupParams p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.x = x; p.ldx = ldx; p.x_vec = x_vec; p.a_scale_out = scales; p.Ka = (int)K;
    p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)(ws + L.off_ws); p.w_scale = w_one; p.w_rows = w_rows;
    p.M = (int)M; p.K = (int)K; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
    p.Jlog = pl.Jlog; p.S = pl.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
    p.stages_total = d.stages_total; p.stages_per_split = d.stages_per_split;
    p.total_tiles = d.total; p.per_xcd = d.per_xcd;
    int rc = d.need32 ? launch_lookup_r<true>(pl.R, pl.BW, kFusedQuant, p, s)
                      : launch_lookup_r<false>(pl.R, pl.BW, kFusedQuant, p, s);
    if (rc != VLUT_OK) return rc;
    if (pl.S > 1) {
        rc = launch_splitk_reduce((const int32_t*)(ws + L.off_ws), pl.S, M, N, w_one, w_rows, (const float*)scales, y, ldy,
                                  acc_or_null, s);
        if (rc != VLUT_OK) return rc;
    }
    return VLUT_OK;
}

// ---- 1.60-bit packing (g = 5)
size_t vlut_packed_weight_bytes_g5(int64_t M, int64_t K) {
    if (!shape5_ok(M, K, 1)) return 0;
    return (size_t)((M + 3) / 4) * (size_t)((K / 5 + 15) / 16) * 64;
}

size_t vlut_packed_offset_g5(int64_t M, int64_t K, int64_t m, int64_t kg) {
    if (!shape5_ok(M, K, 1) || m < 0 || m >= M || kg < 0 || kg >= K / 5) return (size_t)-1;
    size_t KCn = (size_t)((K / 5 + 15) / 16);
    return (((size_t)(m / 4) * KCn + (size_t)(kg / 16)) * 64) + (size_t)(m % 4) * 16 + (size_t)(kg % 16);
}

int vlut_pack_weights_g5(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                         void* stream) {
    if (!shape5_ok(M, K, 1)) return VLUT_ERR_SHAPE;
    if (!w_ternary || !packed) return VLUT_ERR_NULL;
    size_t need = vlut_packed_weight_bytes_g5(M, K);
    if (packed_bytes < need) return VLUT_ERR_SMALL_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_pack_mutex);
    int zero = 0;
    if (hipMemcpyToSymbolAsync(HIP_SYMBOL(g_pack_error), &zero, sizeof(int), 0, hipMemcpyHostToDevice, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    int G = (int)(K / 5), KCn = (G + 15) / 16, RGtotal = (int)((M + 3) / 4);
    size_t blocks = (need + 255) / 256;
    hipLaunchKernelGGL(pack_kernel<5>, dim3((unsigned)blocks), dim3(256), 0, s, w_ternary, (int)M, K, G, KCn, RGtotal,
                       packed);
    if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    int err = 0;
    if (hipMemcpyFromSymbolAsync(&err, HIP_SYMBOL(g_pack_error), sizeof(int), 0, hipMemcpyDeviceToHost, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return VLUT_ERR_DEVICE;
    return err ? VLUT_ERR_VALUE : VLUT_OK;
}

size_t vlut_workspace_bytes_g5(int64_t M, int64_t K, int64_t N) {
    if (!shape5_ok(M, K, N)) return 0;
    Plan5 pl = choose_plan5(M, K, N);
    return pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
}

int vlut_set_plan_g5(int R, int split_k) {
    if (R != 0) {
        bool ok = false;
        for (int v : kSupportedR5) ok = ok || v == R;
        if (!ok) return VLUT_ERR_UNSUPPORTED;
    }
    if (split_k < 0 || split_k > 16) return VLUT_ERR_UNSUPPORTED;
    t_forced5 = {R, split_k};
    return VLUT_OK;
}

int vlut_query_plan_g5(int64_t M, int64_t K, int64_t N, int* out3) {
    if (!out3) return VLUT_ERR_NULL;
    if (!shape5_ok(M, K, N)) return VLUT_ERR_SHAPE;
    Plan5 pl = choose_plan5(M, K, N);
    if (!plan5_valid(pl, M, K, N)) return VLUT_ERR_UNSUPPORTED;   // the override does not fit this shape
    Derived5 d = derive5(pl, M, K, N);
    out3[0] = pl.R; out3[1] = pl.S; out3[2] = d.total;
    return VLUT_OK;
}

int vlut_mpgemm_g5(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                   int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* workspace, size_t workspace_bytes,
                   void* stream) {
    if (!shape5_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !a_q || !a_scale) return VLUT_ERR_NULL;
    if (!y && !acc_or_null) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    if (((uintptr_t)a_q) % 8 != 0) return VLUT_ERR_UNSUPPORTED;       // 5 rows x 8 tokens are read 8 bytes at a time
    Plan5 pl = choose_plan5(M, K, N);
    if (!plan5_valid(pl, M, K, N)) return VLUT_ERR_UNSUPPORTED;
    Derived5 d = derive5(pl, M, K, N);
    size_t ws_need = pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
    if (ws_need > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < ws_need) return VLUT_ERR_SMALL_BUFFER;
    }
    Lookup5Params p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)workspace;
    p.w_scale = w_scale;
    p.M = (int)M; p.K = (int)K; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
    p.S = pl.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
    p.dstages_total = d.dstages_total; p.dstages_per_split = d.dstages_per_split;
    p.total_tiles = d.total; p.per_xcd = d.per_xcd;
    p.Ka = (int)K;
    hipStream_t s = (hipStream_t)stream;
    int grid = d.per_xcd * 8;
    int rc = d.need32 ? launch_lookup5_r<true>(pl.R, p, grid, s) : launch_lookup5_r<false>(pl.R, p, grid, s);
    if (rc != VLUT_OK) return rc;
    if (pl.S > 1)
        return launch_splitk_reduce((const int32_t*)workspace, pl.S, M, N, w_scale, nullptr, a_scale, y, ldy, acc_or_null, s);
    return VLUT_OK;
}

// ---- mixed 1.60-bit / 2-bit packing (Sec. 3.3 "Flexible sub-2-bit weight packing")
int64_t vlut_mixed_k5(int64_t K) {
    if (K < 4 || (K % 4) != 0) return -1;
    return (K / 20) * 20;
}

size_t vlut_packed_weight_bytes_mixed(int64_t M, int64_t K) {
    if (!shape_ok(M, K, 1)) return 0;
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    return (K5 > 0 ? vlut_packed_weight_bytes_g5(M, K5) : 0) + (K4 > 0 ? vlut_packed_weight_bytes(M, K4) : 0);
}

int vlut_pack_weights_mixed(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                            void* stream) {
    if (!shape_ok(M, K, 1)) return VLUT_ERR_SHAPE;
    if (!w_ternary || !packed) return VLUT_ERR_NULL;
    if (packed_bytes < vlut_packed_weight_bytes_mixed(M, K)) return VLUT_ERR_SMALL_BUFFER;
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    const size_t bytes5 = K5 > 0 ? vlut_packed_weight_bytes_g5(M, K5) : 0;
    const size_t bytes4 = K4 > 0 ? vlut_packed_weight_bytes(M, K4) : 0;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_pack_mutex);
    int zero = 0;
    if (hipMemcpyToSymbolAsync(HIP_SYMBOL(g_pack_error), &zero, sizeof(int), 0, hipMemcpyHostToDevice, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    const int RGtotal = (int)((M + 3) / 4);
    if (K5 > 0) {
        const int G = (int)(K5 / 5), KCn = (G + 15) / 16;
        hipLaunchKernelGGL(pack_kernel<5>, dim3((unsigned)((bytes5 + 255) / 256)), dim3(256), 0, s, w_ternary, (int)M, K, G,
                           KCn, RGtotal, packed);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    if (K4 > 0) {
        const int G = (int)(K4 / 4), KCn = (G + 15) / 16;
        hipLaunchKernelGGL(pack_kernel<4>, dim3((unsigned)((bytes4 + 255) / 256)), dim3(256), 0, s, w_ternary + K5, (int)M, K,
                           G, KCn, RGtotal, packed + bytes5);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    int err = 0;
    if (hipMemcpyFromSymbolAsync(&err, HIP_SYMBOL(g_pack_error), sizeof(int), 0, hipMemcpyDeviceToHost, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return VLUT_ERR_DEVICE;
    return err ? VLUT_ERR_VALUE : VLUT_OK;
}

// The two parts as launches of the kernels above in partial-sum mode, then one exact INT32 sum + scale step.
// Workspace: [S5 + S4][N][M] INT32.
static bool mixed_plans(int64_t M, int64_t K, int64_t N, Plan5* p5, Plan* p4) {
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    if (K5 > 0) {
        *p5 = choose_plan5(M, K5, N);
        if (!plan5_valid(*p5, M, K5, N)) return false;
    } else {
        *p5 = Plan5{0, 0};
    }
    *p4 = K4 > 0 ? choose_plan(M, K4, N) : Plan{0, 0, 0, 0};
    if (K4 > 0 && p4->R == 0) return false;              // the override of vlut_set_plan does not fit the 2-bit part
    return true;
}

size_t vlut_workspace_bytes_mixed(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    Plan5 p5;
    Plan p4;
    if (!mixed_plans(M, K, N, &p5, &p4)) return 0;
    return (size_t)(p5.S + p4.S) * (size_t)M * (size_t)N * sizeof(int32_t);
}

int vlut_mpgemm_mixed(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                      int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* workspace, size_t workspace_bytes,
                      void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    if (((uintptr_t)a_q) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    Plan5 pl5;
    Plan pl4;
    if (!mixed_plans(M, K, N, &pl5, &pl4)) return VLUT_ERR_UNSUPPORTED;
    const size_t need = (size_t)(pl5.S + pl4.S) * (size_t)M * (size_t)N * sizeof(int32_t);
    if (!workspace) return VLUT_ERR_NULL;
    if (workspace_bytes < need) return VLUT_ERR_SMALL_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    if (K5 > 0) {
        const Derived5 d = derive5(pl5, M, K5, N);
        Lookup5Params p;
        std::memset(&p, 0, sizeof(p));
        p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.ws = (int32_t*)workspace; p.w_scale = w_scale;
        p.M = (int)M; p.K = (int)K5; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
        p.S = pl5.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
        p.dstages_total = d.dstages_total; p.dstages_per_split = d.dstages_per_split;
        p.total_tiles = d.total; p.per_xcd = d.per_xcd;
        p.Ka = (int)K; p.partial = 1;
        const int grid = d.per_xcd * 8;
        rc = d.need32 ? launch_lookup5_r<true>(pl5.R, p, grid, s) : launch_lookup5_r<false>(pl5.R, p, grid, s);
        if (rc != VLUT_OK) return rc;
    }
    if (K4 > 0) {
        const Derived d = derive(pl4, M, K4, N);
        LookupParams p;
        std::memset(&p, 0, sizeof(p));
        p.packed = packed + (K5 > 0 ? vlut_packed_weight_bytes_g5(M, K5) : 0);
        p.a_q = a_q + (size_t)K5 * 8;                      // activation rows K5 .. K-1 of every token chunk
        p.a_scale = a_scale; p.ws = (int32_t*)workspace; p.w_scale = w_scale;
        p.M = (int)M; p.K = (int)K4; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
        p.Jlog = pl4.Jlog; p.S = pl4.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
        p.stages_total = d.stages_total; p.stages_per_split = d.stages_per_split;
        p.total_tiles = d.total; p.per_xcd = d.per_xcd;
        p.Ka = (int)K; p.partial = 1; p.slot0 = pl5.S;
        rc = d.need32 ? launch_lookup_r<true>(pl4.R, pl4.BW, kFast, p, s) : launch_lookup_r<false>(pl4.R, pl4.BW, kFast, p, s);
        if (rc != VLUT_OK) return rc;
    }
    return launch_splitk_reduce((const int32_t*)workspace, pl5.S + pl4.S, M, N, w_scale, nullptr, a_scale, y, ldy,
                                acc_or_null, s);
}

size_t vlut_mfma_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    const MfmaPlan mp = mfma_plan(M, K, N);
    return mp.S > 1 ? (size_t)mp.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
}

int vlut_mpgemm_mfma(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale,
                     const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                     int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    if (lut_or_null) return VLUT_ERR_UNSUPPORTED;
    if (((uintptr_t)a_q) % 16 != 0 || ((uintptr_t)packed) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    const MfmaPlan mp = mfma_plan(M, K, N);
    const size_t need = mp.S > 1 ? (size_t)mp.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
    if (need > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < need) return VLUT_ERR_SMALL_BUFFER;
        if (((uintptr_t)workspace) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    }
    hipStream_t s = (hipStream_t)stream;
    MfmaParams p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)workspace;
    p.w_scale = w_scale; p.M = (int)M; p.K = (int)K; p.N = (int)N;
    p.KCn = (int)((K / 4 + 15) / 16); p.RGtotal = (int)((M + 3) / 4); p.ldy = (int)ldy; p.chunks = (int)((N + 7) / 8);
    p.S = mp.S; p.steps_per_split = mp.steps_per_split; p.tiles_m = mp.tiles_m; p.tiles_n = mp.tiles_n;
    if (mp.S > 1) p.out_vec = (M % 4 == 0) ? 1 : 0;
    else p.out_vec = (!y || (((uintptr_t)y % 16 == 0) && (ldy % 4 == 0))) ? 1 : 0;
    const dim3 grid((unsigned)mp.grid);
    switch (mp.BN) {
    case 128: hipLaunchKernelGGL(mfma_kernel<128>, grid, dim3(256), 0, s, p); break;
    case 64: hipLaunchKernelGGL(mfma_kernel<64>, grid, dim3(256), 0, s, p); break;
    case 32: hipLaunchKernelGGL(mfma_kernel<32>, grid, dim3(256), 0, s, p); break;
    default: hipLaunchKernelGGL(mfma_kernel<16>, grid, dim3(256), 0, s, p); break;
    }
    if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    if (mp.S > 1)
        return launch_splitk_reduce((const int32_t*)workspace, mp.S, M, N, w_scale, nullptr, a_scale, y, ldy, acc_or_null, s);
    return VLUT_OK;
}

}  // extern "C"
