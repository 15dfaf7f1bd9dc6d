// K2 / K4 -- the two matrix products of the HLQ backward pass (arXiv 2406.15102, Sec. 6.1), one
// launch per product: the kernel around the tile body of gemm_body.hpp, the split-K reduction, the
// plan (tile size, k splits) and the host-side dispatch over the template arguments.
#include "gemm_body.hpp"
#include "gemm_dl_body.hpp"
#include "gemm_plan.hpp"
#include "reduce_body.hpp"

#include <atomic>

namespace hlq {

// operands straight into LDS (gemm_dl_body.hpp) wherever the shape allows; switched off for A/B runs
static std::atomic<int> g_dl_enabled{1};
void gemm_dl_enable(bool on) { g_dl_enabled.store(on ? 1 : 0); }
bool gemm_dl_ok(int Kb, int splits)
{
    // whole 128-byte steps, and enough of them per workgroup to fill the ring's pipeline
    return g_dl_enabled.load() != 0 && Kb % 128 == 0 && (Kb / 128) / splits >= 4;
}

// `gt`: the product's last rows in 192-row tiles (gt.tiles_m = 0: none), dispatched behind the n_main
// workgroups of the 256-row tiles
template <int KIND, int OUT>
__global__ __launch_bounds__(256) void k_gemm_dl(GemmDev g, GemmDev gt, int n_main)
{
    const int b = static_cast<int>(blockIdx.x);
    if constexpr (KIND != 2 && OUT != 2 && OUT != 3) {
        if (b >= n_main) {
            gemm_tile_dl<KIND, 6, OUT>(gt, b - n_main);
            return;
        }
    }
    gemm_tile_dl<KIND, 8, OUT>(g, b);
}

template <int KIND, int WM, int WN, int KCH, bool TAIL, int OUT>
__global__ __launch_bounds__(256) void k_gemm_nt(GemmDev g)
{
    gemm_tile<KIND, WM, WN, KCH, TAIL, OUT>(g, static_cast<int>(blockIdx.x));
}

// ---- split-K: the reduction of the partial accumulators as a kernel of its own (reduce_body.hpp) ----
template <int KIND, bool F32>
__global__ __launch_bounds__(256) void k_splitk_reduce(const int32_t *__restrict__ partial, int splits, int M, int N,
                                                       const float *__restrict__ sA, const float *__restrict__ sB,
                                                       float alpha, void *__restrict__ C)
{
    splitk_reduce_body<KIND, F32>(partial, splits, M, N, sA, sB, alpha, C, blockIdx.x);
}

// `nk` = k steps of the product (128 B of k per operand row);
// `scale` = cost of such a step relative to the byte-operand kernels.
GemmPlan plan_gemm(int M, int N, int nk, double scale, size_t ws_bytes, bool allow_split)
{
    const double mn = static_cast<double>(M) * N;
    GemmPlan best{true, 1};
    double best_t = 1e30;
    for (int big = 1; big >= 0; --big) {
        const int tile = big ? 256 : 128;
        const double tiles = static_cast<double>((M + tile - 1) / tile) * ((N + tile - 1) / tile);
        const double slots = big ? 256.0 : 512.0, fixed = big ? 12.0 : 6.0;
        for (int S = 1; S <= 16; ++S) {
            // two co-resident 128-tile workgroups share a compute unit's LDS and power: slower steps
            const double step = scale * (big ? 1.6 : (tiles * S > 256.0 ? 0.95 : 0.5));
            if (S > 1 && (!allow_split || S > nk || static_cast<double>(S) * mn * 4.0 > static_cast<double>(ws_bytes))) break;
            const double rounds = __builtin_ceil(tiles * S / slots);
            double t = rounds * (__builtin_ceil(static_cast<double>(nk) / S) * step + fixed);
            if (S > 1) t += 2.0 * S * mn * 4.0 / 5.0e6 + 4.0;
            if (t < best_t) { best_t = t; best = GemmPlan{big != 0, S}; }
        }
    }
    return best;
}

// the last rows of a product in 192-row tiles where that saves a quarter of its last round (gemm_plan.hpp)
static std::atomic<int> g_tail_enabled{1};
void gemm_tail_enable(bool on) { g_tail_enabled.store(on ? 1 : 0); }
bool gemm_tail_enabled() { return g_tail_enabled.load() != 0; }

// plan overrides for measurements (hlq_set_option): 0 = the cost model decides
static std::atomic<int> g_plan_tile{0}, g_plan_splits{0};
void gemm_plan_force(int tile, int splits)
{
    if (tile >= 0) g_plan_tile.store(tile);
    if (splits >= 0) g_plan_splits.store(splits);
}
int gemm_plan_forced_tile() { return g_plan_tile.load(); }
// the forced k split, cut down to what the reduction (nk steps) and the scratch (bytes for M x N partials) allow
int gemm_plan_forced_splits(int nk, double mn, size_t ws_bytes, bool allow_split)
{
    int S = g_plan_splits.load();
    if (S <= 0) return 0;
    if (!allow_split) return 1;
    if (S > 16) S = 16;
    if (S > nk) S = nk;
    while (S > 1 && static_cast<double>(S) * mn * 4.0 > static_cast<double>(ws_bytes)) --S;
    return S < 1 ? 1 : S;
}

GemmPlan plan_for(int kind, int M, int N, int K, size_t ws_bytes, bool allow_split)
{
    // a step of the packed product carries twice the MFMAs of a byte-operand step
    const int nk = (row_bytes(kind, K) + 127) / 128;
    GemmPlan p = plan_gemm(M, N, nk, kind == 2 ? P4_STEP_SCALE : 1.0, ws_bytes, allow_split);
    if (const int t = gemm_plan_forced_tile()) p.big = t == 256;
    if (const int S = gemm_plan_forced_splits(nk, static_cast<double>(M) * N, ws_bytes, allow_split)) p.splits = S;
    return p;
}

size_t gemm_ws_bytes(int kind, int M, int N, int K)
{
    const GemmPlan p = plan_for(kind, M, N, K, ~static_cast<size_t>(0), true);
    return p.splits > 1 ? static_cast<size_t>(p.splits) * M * N * 4 : 0;
}

SplitReduce splitk_reduce_job_of(int kind, const GemmArgs &a, int splits)
{
    const int64_t quads = (static_cast<int64_t>(a.M) * a.N + 3) / 4;
    return SplitReduce{static_cast<const int32_t *>(a.ws), splits, a.M, a.N, a.sA, a.sB, a.alpha, a.C, kind, a.c_is_f32 ? 1 : 0,
                       static_cast<int>((quads + 255) / 256)};
}

// kind 0: int32 partials (the two integer products), kind 1: fp32 partials
hipError_t launch_splitk_reduce(int kind, const GemmArgs &a, int splits, hipStream_t st)
{
    const int64_t quads = (static_cast<int64_t>(a.M) * a.N + 3) / 4;
    const unsigned grid = static_cast<unsigned>((quads + 255) / 256);
    const int32_t *part = static_cast<const int32_t *>(a.ws);
#define HLQ_REDUCE(KIND, F32) \
    hipLaunchKernelGGL((k_splitk_reduce<KIND, F32>), dim3(grid), dim3(256), 0, st, part, splits, a.M, a.N, a.sA, a.sB, a.alpha, a.C)
    if (kind == 0) {
        if (a.c_is_f32) HLQ_REDUCE(0, true); else HLQ_REDUCE(0, false);
    } else {
        if (a.c_is_f32) HLQ_REDUCE(1, true); else HLQ_REDUCE(1, false);
    }
#undef HLQ_REDUCE
    return hipGetLastError();
}

template <int KIND, int WM, int WN, int KCH, bool TAIL, int OUT>
static hipError_t launch_tt(const GemmArgs &a, int splits, hipStream_t st)
{
    const GemmDev g = gemm_dev(KIND, a, 64 * WM, 64 * WN, splits);
    constexpr size_t lds_bytes = gemm_lds_bytes(WM, WN, KCH);
    static bool attr_set = false;     // raising the dynamic-LDS limit is idempotent; racing callers set the same value
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_nt<KIND, WM, WN, KCH, TAIL, OUT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_gemm_nt<KIND, WM, WN, KCH, TAIL, OUT>), dim3(g.tiles_m * g.tiles_n * splits), dim3(256), lds_bytes, st, g);
    return hipGetLastError();
}

template <int KIND, int OUT>
static hipError_t launch_dl(const GemmArgs &a, int splits, hipStream_t st)
{
    GemmDev g = gemm_dev(KIND, a, 256, 256, splits);
    GemmDev gt = g;
    gt.tiles_m = 0;
    if (KIND != 2 && (OUT == 0 || OUT == 1) && splits == 1) {
        const int tail_rows = gemm_tail_rows(a.M, a.N, 0);
        if (tail_rows > 0) gt = gemm_dev_cut_tail(g, tail_rows);
    }
    static bool attr_set = false;     // idempotent; racing callers set the same value
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_dl<KIND, OUT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kGemmDlLdsBytes));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int n_main = g.tiles_m * g.tiles_n * splits, n_tail = gt.tiles_m * gt.tiles_n;
    hipLaunchKernelGGL((k_gemm_dl<KIND, OUT>), dim3(n_main + n_tail), dim3(256), kGemmDlLdsBytes, st, g, gt, n_main);
    return hipGetLastError();
}

template <int KIND, int WM, int WN, int KCH, int OUT>
static hipError_t launch_o(const GemmArgs &a, int splits, hipStream_t st)
{
    const int Kb = row_bytes(KIND, a.K);
    if (WM == 4 && WN == 4 && gemm_dl_ok(Kb, splits)) return launch_dl<KIND, OUT>(a, splits, st);
    return (Kb % (KCH * 16) == 0) ? launch_tt<KIND, WM, WN, KCH, false, OUT>(a, splits, st)
                                  : launch_tt<KIND, WM, WN, KCH, true, OUT>(a, splits, st);
}

template <int KIND, int WM, int WN, int KCH>
static hipError_t launch_t(const GemmArgs &a, int splits, hipStream_t st)
{
    // the raw accumulators and the scaled output are separate launches of the same product
    if (KIND != 1 && a.acc) {
        hipError_t e = launch_o<KIND, WM, WN, KCH, 2>(a, 1, st);
        if (e != hipSuccess || !a.C) return e;
    }
    if (splits > 1) {
        hipError_t e = launch_o<KIND, WM, WN, KCH, 3>(a, splits, st);
        if (e != hipSuccess) return e;
        return launch_splitk_reduce(KIND == 1 ? 1 : 0, a, splits, st);
    }
    return a.c_is_f32 ? launch_o<KIND, WM, WN, KCH, 1>(a, 1, st) : launch_o<KIND, WM, WN, KCH, 0>(a, 1, st);
}

hipError_t launch_gemm_nt(int kind, const GemmArgs &a, hipStream_t st)
{
    const bool can_split = a.ws != nullptr && a.C != nullptr && (reinterpret_cast<uintptr_t>(a.ws) & 15) == 0;
    const GemmPlan p = plan_for(kind, a.M, a.N, a.K, a.ws_bytes, can_split);
    if (p.big && p.splits == 1 && gemm_stream_wanted(kind, a, 0, nullptr)) return launch_gemm_stream(kind, a, 0, nullptr, st);
    if (kind == 0) return p.big ? launch_t<0, 4, 4, 8>(a, p.splits, st) : launch_t<0, 2, 2, 8>(a, p.splits, st);
    if (kind == 2) return p.big ? launch_t<2, 4, 4, 8>(a, p.splits, st) : launch_t<2, 2, 2, 8>(a, p.splits, st);
    return p.big ? launch_t<1, 4, 4, 8>(a, p.splits, st) : launch_t<1, 2, 2, 8>(a, p.splits, st);
}

}  // namespace hlq
