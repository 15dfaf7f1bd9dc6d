// Host-side planning shared by the launchers of the matrix products (k_gemm.hip, k_gemm_pair.hip).
#pragma once
#include "gemm_common.hpp"

namespace hlq {

// bytes per operand row: int8 codes, bf16 values, nibble-packed codes
static inline int row_bytes(int kind, int K) { return kind == 0 ? K : (kind == 1 ? 2 * K : K / 2); }

// Plan: tile size and number of k splits, from a small cost model (microseconds) fitted to
// measurements on MI355X: a 256-tile step (128 B of k) costs ~1.6 us and a tile ~12 us of fixed
// prologue/epilogue, one workgroup per compute unit; a 128-tile step ~0.5 us alone on its compute
// unit and ~0.95 us when two share it, ~6 us fixed; the split-K partials cost their HBM round trip
// plus a launch.  A step of the packed product carries twice the MFMAs of a byte-operand step.
constexpr double P4_STEP_SCALE = 1.8;
struct GemmPlan {
    bool big;
    int splits;
};
// `nk` = k steps of the product (128 B of k per operand row); `scale` = cost of such a step relative
// to the byte-operand kernels.
GemmPlan plan_gemm(int M, int N, int nk, double scale, size_t ws_bytes, bool allow_split);
GemmPlan plan_for(int kind, int M, int N, int K, size_t ws_bytes, bool allow_split);

// measurement overrides of the plans (hlq_set_option): tile = 0 (the model decides), 128 or 256 for every
// product; splits = 0 (the model decides) or the k split of a single product / of the g_w product of a
// pair, cut down to what the reduction and the scratch allow.  A negative argument leaves that setting.
void gemm_plan_force(int tile, int splits);
int gemm_plan_forced_tile();
int gemm_plan_forced_splits(int nk, double mn, size_t ws_bytes, bool allow_split);

// whether a 256-tiled product with rows of Kb bytes, its k split `splits` ways, takes the kernel that
// loads its operands straight into LDS (gemm_dl_body.hpp)
bool gemm_dl_ok(int Kb, int splits);
void gemm_dl_enable(bool on);

// kernel argument block of one product tiled BM x BN, k split `splits` ways
static inline GemmDev gemm_dev(int kind, const GemmArgs &a, int BM, int BN, int splits)
{
    GemmDev g;
    g.A = static_cast<const char *>(a.A);
    g.Bm = static_cast<const char *>(a.Bm);
    g.M = a.M;
    g.N = a.N;
    g.Kb = row_bytes(kind, a.K);
    g.sA = a.sA;
    g.sB = a.sB;
    g.alpha = a.alpha;
    g.C = a.C;
    g.c_is_f32 = a.c_is_f32 ? 1 : 0;
    g.acc = a.acc;
    g.tiles_m = (a.M + BM - 1) / BM;
    g.tiles_n = (a.N + BN - 1) / BN;
    g.splits = splits;
    g.partial = static_cast<int32_t *>(a.ws);
    return g;
}

// dynamic LDS of a workgroup: two operand stages, or the four epilogue slabs if those are larger
constexpr size_t gemm_lds_bytes(int WM, int WN, int KCH)
{
    const size_t main_bytes = 2u * (64 * WM + 64 * WN) * KCH * 16u;
    const size_t epi_bytes = 4u * (32u * (32u * WN * 4u + 16u));
    return main_bytes > epi_bytes ? main_bytes : epi_bytes;
}

}  // namespace hlq
