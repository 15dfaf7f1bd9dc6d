// K2 | K4 in one launch: the plan and the dispatch over the operand kinds.  The kernels live in
// gemm_pair_impl.hpp, instantiated by k_gemm_pair_KK.hip for KK = (kind of the g_x product, kind of
// the g_w product): 21 the default lists (packed 4-bit codes, bf16 projections), 20 with the integer
// g_w list, 01 / 00 the same with one int8 per g_x code (8-bit warm-up, unpacked storage).
#include "gemm_plan.hpp"

namespace hlq {

hipError_t launch_pair_21(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigA, bool f32, bool bigB, int outB,
                          bool b_first, hipStream_t st);
hipError_t launch_pair_20(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigA, bool f32, bool bigB, int outB,
                          bool b_first, hipStream_t st);
hipError_t launch_pair_01(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigA, bool f32, bool bigB, int outB,
                          bool b_first, hipStream_t st);
hipError_t launch_pair_00(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigA, bool f32, bool bigB, int outB,
                          bool b_first, hipStream_t st);

// Plan of the pair: tile size of either product and the k split of the g_w product, by a model of
// how the launch unfolds (microseconds; constants fitted to a sweep of every plan, either dispatch
// order, over thirteen layer shapes on MI355X).  A tile of nk steps (128 B of k) takes nk * step + fixed.  A 256-tile owns a
// compute unit.  128-tiles share one in twos only if both products use them (the launch has one LDS
// size, the larger) and there are more of them than compute units; they step faster alone.
// Workgroups are dispatched in index order, one product's tiles then the other's (both orders are
// priced), each to the first free slot: after the first product's full rounds, the slots of its last, partial round free up one
// tile later than the rest, and the other product's tiles -- all equal -- finish at the first instant
// by which enough of them fit.
struct PairPlan {
    bool bigA, bigB;
    int splitsB;
    bool b_first;    // the g_w product's tiles are dispatched first
};

namespace {
constexpr double kStepBig = 1.3, kPackedScale = 1.8, kStepSmallAlone = 0.6, kStepSmallShared = 0.9;
constexpr double kFixedBig = 16.0, kFixedSmall = 6.5;
constexpr double kOneStepSaves = 2.0;    // a tile of one step skips the pipeline (gemm_body.hpp)
constexpr int kSplitChoices[] = {1, 2, 3, 4, 6, 8, 12, 16};

struct TileClass {
    double step, fixed;
    int slots;   // tiles in flight on the chip
};
TileClass tile_class(bool big, bool mixed, double n)
{
    if (big) return {kStepBig, kFixedBig, 256};
    if (mixed || n <= 256.0) return {kStepSmallAlone, kFixedSmall, 256};
    return {kStepSmallShared, kFixedSmall, 512};
}

// nA tiles of tA on mA slots, then nB tiles of tB on mB slots (the same silicon, possibly cut finer)
double pair_makespan(double nA, double tA, int mA, double nB, double tB, int mB)
{
    const double qA = __builtin_floor(nA / mA), rA = nA - qA * mA;
    const double T1 = qA * tA, T2 = rA > 0 ? T1 + tA : T1;
    const double g2 = __builtin_round(rA / mA * mB), g1 = mB - g2;      // slots free at T2 / at T1
    // candidate finishing times: T1 + k tB and T2 + k tB; the first with enough capacity
    double best = 1e30;
    for (int grp = 0; grp < 2; ++grp) {
        const double base = grp ? T2 : T1;
        const double gs = grp ? g2 : g1;
        if (gs <= 0) continue;
        // smallest k with g1 floor((T - T1)/tB) + g2 floor((T - T2)/tB) >= nB at T = base + k tB
        double lo = grp ? 0 : 1, hi = __builtin_ceil(nB / gs) + 1;
        while (lo < hi) {
            const double k = __builtin_floor((lo + hi) / 2), T = base + k * tB;
            const double c1 = g1 * __builtin_fmax(0.0, __builtin_floor((T - T1) / tB + 1e-9));
            const double c2 = g2 * __builtin_fmax(0.0, __builtin_floor((T - T2) / tB + 1e-9));
            if (c1 + c2 >= nB) hi = k; else lo = k + 1;
        }
        const double T = base + lo * tB;
        if (T < best) best = T;
    }
    return best > T2 ? best : T2;
}
}  // namespace

static PairPlan plan_pair(const GemmArgs &a, int kindA, const GemmArgs &b, int kindB, size_t ws_bytes)
{
    const int nkA = (row_bytes(kindA, a.K) + 127) / 128, nkB = (row_bytes(kindB, b.K) + 127) / 128;
    const double scaleA = kindA == 2 ? kPackedScale : 1.0, scaleB = kindB == 2 ? kPackedScale : 1.0;
    const double mnB = static_cast<double>(b.M) * b.N;
    PairPlan best{true, true, 1, false};
    double best_t = 1e30;
    for (int bigA = 1; bigA >= 0; --bigA) {
        for (int bigB = 1; bigB >= 0; --bigB) {
            const bool mixed = bigA != bigB;
            const int ta = bigA ? 256 : 128, tb = bigB ? 256 : 128;
            const double nA = static_cast<double>((a.M + ta - 1) / ta) * ((a.N + ta - 1) / ta);
            const double nB1 = static_cast<double>((b.M + tb - 1) / tb) * ((b.N + tb - 1) / tb);
            const TileClass ca = tile_class(bigA != 0, mixed, nA);
            const double tA = nkA * scaleA * ca.step + ca.fixed - (nkA == 1 ? kOneStepSaves : 0.0);
            for (int S : kSplitChoices) {
                if (S > 1 && (S > nkB || S * mnB * 4.0 > static_cast<double>(ws_bytes))) break;
                const TileClass cb = tile_class(bigB != 0, mixed, nB1 * S);
                const double stepsB = __builtin_ceil(static_cast<double>(nkB) / S);
                const double tB = stepsB * scaleB * cb.step + cb.fixed - (stepsB == 1.0 ? kOneStepSaves : 0.0);
                // either product may go first: usually the one with the longer tiles, which must not start late
                const double tab = pair_makespan(nA, tA, ca.slots, nB1 * S, tB, cb.slots);
                const double tba = pair_makespan(nB1 * S, tB, cb.slots, nA, tA, ca.slots);
                const bool b_first = tba < tab;
                double t = b_first ? tba : tab;
                if (S > 1) t += 2.0 * S * mnB * 4.0 / 8.0e6 + 3.0;     // partials out and back, one more launch
                if (t < best_t) {
                    best_t = t;
                    best = PairPlan{bigA != 0, bigB != 0, S, b_first};
                }
            }
        }
    }
    if (const int t = gemm_plan_forced_tile()) best.bigA = best.bigB = t == 256;
    if (const int S = gemm_plan_forced_splits(nkB, mnB, ws_bytes, ws_bytes > 0)) best.splitsB = S;
    return best;
}

// split-k scratch the pair's plan asks for when it may have up to `cap` bytes
size_t gemm_pair_ws_bytes(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b, size_t cap)
{
    const PairPlan p = plan_pair(a, kindA, b, kindB, cap);
    return p.splitsB > 1 ? static_cast<size_t>(p.splitsB) * b.M * b.N * 4 : 0;
}

void gemm_pair_describe(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b, size_t ws_bytes, int plan[5])
{
    const PairPlan p = plan_pair(a, kindA, b, kindB, ws_bytes);
    plan[0] = p.bigA ? 256 : 128;
    plan[1] = p.bigB ? 256 : 128;
    plan[2] = p.splitsB;
    plan[3] = p.b_first ? 1 : 0;
    plan[4] = (p.bigA && p.bigB && p.splitsB == 1 && gemm_stream_wanted(kindA, a, kindB, &b)) ? 1 : 0;
}

bool gemm_pair_available(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b)
{
    // the grid of the launch (128-tiles of both products, the second split 16 ways) must fit 31 bits with room
    const int64_t blocks = static_cast<int64_t>((a.M + 127) / 128) * ((a.N + 127) / 128) +
                           16 * static_cast<int64_t>((b.M + 127) / 128) * ((b.N + 127) / 128);
    return (kindA == 2 || kindA == 0) && (kindB == 1 || kindB == 0) && a.C && b.C && !a.acc && !b.acc &&
           a.c_is_f32 == b.c_is_f32 && blocks < (int64_t(1) << 30);
}

hipError_t launch_gemm_pair(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b, hipStream_t st, SplitReduce *defer)
{
    if (defer) defer->blocks = 0;
    if (!gemm_pair_available(kindA, a, kindB, b)) return hipErrorInvalidValue;
    const bool can_split = b.ws != nullptr && (reinterpret_cast<uintptr_t>(b.ws) & 15) == 0;
    const PairPlan p = plan_pair(a, kindA, b, kindB, can_split ? b.ws_bytes : 0);
    if (p.bigA && p.bigB && p.splitsB == 1 && gemm_stream_wanted(kindA, a, kindB, &b))
        return launch_gemm_stream(kindA, a, kindB, &b, st);
    const GemmDev ga = gemm_dev(kindA, a, p.bigA ? 256 : 128, p.bigA ? 256 : 128, 1);
    GemmDev gb = gemm_dev(kindB, b, p.bigB ? 256 : 128, p.bigB ? 256 : 128, p.splitsB);
    const int outB = p.splitsB > 1 ? 3 : (b.c_is_f32 ? 1 : 0);
    // the g_w product's last rows in 192-row tiles when it closes the launch on 256-tiles that load straight
    // into LDS and its last round would be partly empty (gemm_plan.hpp)
    GemmDev gbt = gb;
    gbt.tiles_m = 0;
    if (p.bigA && p.bigB && p.splitsB == 1 && !p.b_first && kindB != 2 && gemm_dl_ok(gb.Kb, 1)) {
        const int tail_rows = gemm_tail_rows(b.M, b.N, ga.tiles_m * ga.tiles_n);
        if (tail_rows > 0) gbt = gemm_dev_cut_tail(gb, tail_rows);
    }
    hipError_t e;
    if (kindA == 2)
        e = kindB == 1 ? launch_pair_21(ga, gb, gbt, p.bigA, a.c_is_f32, p.bigB, outB, p.b_first, st)
                       : launch_pair_20(ga, gb, gbt, p.bigA, a.c_is_f32, p.bigB, outB, p.b_first, st);
    else
        e = kindB == 1 ? launch_pair_01(ga, gb, gbt, p.bigA, a.c_is_f32, p.bigB, outB, p.b_first, st)
                       : launch_pair_00(ga, gb, gbt, p.bigA, a.c_is_f32, p.bigB, outB, p.b_first, st);
    if (e != hipSuccess || p.splitsB == 1) return e;
    if (defer) {
        *defer = splitk_reduce_job_of(kindB == 1 ? 1 : 0, b, p.splitsB);
        return hipSuccess;
    }
    return launch_splitk_reduce(kindB == 1 ? 1 : 0, b, p.splitsB, st);
}

}  // namespace hlq
