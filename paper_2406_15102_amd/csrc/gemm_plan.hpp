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

// Rows at the end of a product of M x N in 256 x 256 tiles that are better served by 192-row tiles
// (gemm_dl_body.hpp), 0 = none: when `before` tiles of the same launch are dispatched ahead of it and its
// last round on `slots` compute units would be partly empty, the row tiles that reach into that round --
// and as many more as it takes for the rest to fit the full rounds -- are cut into 192-row tiles if those
// then fit one round: the last round shrinks to three quarters.  Switched off by gemm_tail_enable(false).
void gemm_tail_enable(bool on);
bool gemm_tail_enabled();
static inline int gemm_tail_rows(int M, int N, int before, int slots = 256)
{
    if (!gemm_tail_enabled()) return 0;
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    const int64_t total = static_cast<int64_t>(before) + static_cast<int64_t>(tiles_m) * tiles_n;
    const int rem = static_cast<int>(total % slots);
    if (rem == 0 || total < slots) return 0;               // whole rounds, or less than one
    const int64_t cap = total - rem;                          // what the full rounds hold
    const int rt = (rem + tiles_n - 1) / tiles_n;             // row tiles that reach into the last round
    if (rt > tiles_m) return 0;
    const int main_rows = (tiles_m - rt) * 256;
    const int tail_rows = M - main_rows;
    const int64_t main_tiles = static_cast<int64_t>(tiles_m - rt) * tiles_n;
    const int64_t tail_tiles = static_cast<int64_t>((tail_rows + 191) / 192) * tiles_n;
    if (before + main_tiles + tail_tiles > cap + slots) return 0;   // the 192-row tiles would start another round
    return tail_rows;
}

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

// the last `tail_rows` rows of the product `g` (tiled 256 x 256, no k split, output C) as a product of
// its own in tiles of 192 x 256; `g` is cut back to the rows before them
static inline GemmDev gemm_dev_cut_tail(GemmDev &g, int tail_rows)
{
    GemmDev t = g;
    const int main_rows = g.M - tail_rows;
    const int64_t esz = g.c_is_f32 ? 4 : 2;
    t.A = g.A + static_cast<int64_t>(main_rows) * g.Kb;
    t.M = tail_rows;
    t.sA = g.sA ? g.sA + main_rows : nullptr;
    t.C = static_cast<char *>(g.C) + static_cast<int64_t>(main_rows) * g.N * esz;
    t.tiles_m = (tail_rows + 191) / 192;
    g.M = main_rows;
    g.tiles_m = main_rows / 256;
    return t;
}

// dynamic LDS of a workgroup: two operand stages, or the four epilogue slabs if those are larger
constexpr size_t gemm_lds_bytes(int WM, int WN, int KCH)
{
    const size_t main_bytes = 2u * (64 * WM + 64 * WN) * KCH * 16u;
    const size_t epi_bytes = 4u * (32u * (32u * WN * 4u + 16u));
    return main_bytes > epi_bytes ? main_bytes : epi_bytes;
}

}  // namespace hlq
