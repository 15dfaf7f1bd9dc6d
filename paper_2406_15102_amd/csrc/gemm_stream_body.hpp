// Persistent form of K2 / K4 -- the two matrix products of the HLQ backward pass (arXiv 2406.15102,
// Sec. 6.1: stages 5-6 of the g_x list, stage 5 of the g_w list) -- for layers whose products are
// many 256 x 256 tiles per compute unit.
//
// One workgroup per compute unit walks a fixed list of tiles instead of one workgroup per tile.  The
// tile arithmetic is that of gemm_body.hpp (same MFMA order per tile, hence the same bits); what
// changes is what happens between two tiles:
//   * the global loads keep running two k steps ahead ACROSS the tile boundary: while the last two
//     steps of a tile are multiplied, the first two steps of the next tile are loaded; when the tile
//     ends the first of them is staged in LDS and the second is written to the stage the last step
//     has just consumed, so the next tile starts with both LDS stages full -- no prologue latency,
//     and no staged operands held in registers across the epilogue;
//   * the epilogue stages C through LDS of its own (beyond the two operand stages), 16 rows at a
//     time, so it needs no barrier; its stores drain under the next tile's MFMAs;
//   * the first step of a tile stages nothing (both stages are full): by the time the second step
//     needs the registers that the third step's loads fill, those loads -- issued right behind the
//     epilogue's stores -- have had a whole step to land;
//   * no workgroup is retired and dispatched between tiles.
// The schedule is static (tile t of a workgroup is a function of its index alone), so results do
// not depend on timing.  Workgroup w sits on XCD w mod 8 (round-robin dispatch of the first wave of
// workgroups); each XCD owns a contiguous range of the XCD-ordered tile list of gemm_body.hpp and
// its workgroups walk it side by side, so the tiles in flight on one L2 form a compact patch.
// Requirements (checked by the launcher): bf16 output, whole k steps (row bytes a multiple of 128),
// at least four k steps, 256 x 256 tiles, no k split, a grid that is a multiple of 8; dynamic LDS of
// gemm_stream_lds_bytes(): the two operand stages plus the four epilogue areas.
#pragma once
#include "gemm_common.hpp"

namespace hlq {

// Epilogue of one 256 x 256 tile for the persistent kernel: C = alpha * sA[m] * sB[n] * acc in bf16, the
// arithmetic of store_scaled (gemm_common.hpp) value for value, but written to keep few registers
// live and little LDS busy: the column factors alpha * sB[n] of the wavefront's 128 columns wait in
// LDS instead of registers, and the wavefront's 128 x 128 sub-tile is converted, staged and stored
// in pieces of 32 rows x 64 columns (every lane holds part of every piece).  All global accesses are
// buffer instructions on scalar bases with 32-bit lane offsets: no 64-bit pointer arithmetic in
// vector registers, and every load of the epilogue (the scales) is issued before its first store --
// a later load would have to wait for the stores in front of it.
// area: wavefront-private LDS, 512 B of column factors followed by one piece of 32 rows x 144 B.
template <bool V> struct BoolTag { static constexpr bool value = V; };
constexpr int kStreamEpiPitch = 64 * 2 + 16;
constexpr int kStreamEpiBytes = 512 + 32 * kStreamEpiPitch;
// interior: the tile lies inside C and rows of C are 16-byte aligned (no store needs a test).
template <int KIND>
__device__ __forceinline__ void stream_epilogue(typename Mma<KIND>::acc_t (&acc)[4][4], const GemmDev &g, int wm0, int wn0,
                                                int lane, char *area, const bool interior)
{
    constexpr int WM = 4, WN = 4;
    constexpr int PITCH = kStreamEpiPitch;
    const int fr = lane & 31, fh = lane >> 5;
    float *const csl = reinterpret_cast<float *>(area);
    char *const slab = area + 512;
    float sa[WM];
    if (KIND != 1) {
        if (g.sA) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(g.sA), 0, 0x7FFFFFFF, 0x00020000);
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                int m = wm0 + i * 32 + fr;
                m = m < g.M ? m : 0;
                sa[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, m * 4, 0, 0));
            }
        } else {
#pragma unroll
            for (int i = 0; i < WM; ++i) sa[i] = 1.0f;
        }
        if (lane < 32) {
            int n = wn0 + lane * 4;
            n = n < g.N ? n : 0;
            f32x4 v = {g.alpha, g.alpha, g.alpha, g.alpha};
            if (g.sB) {
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(g.sB), 0, 0x7FFFFFFF, 0x00020000);
                v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, n * 4, 0, 0)) * g.alpha;
            }
            *reinterpret_cast<f32x4 *>(csl + lane * 4) = v;
        }
        lds_wave_fence();
    }
    // C rows of this wavefront through one resource at its first row; lane part of the offset in one register
    const __amdgpu_buffer_rsrc_t rsC = __builtin_amdgcn_make_buffer_rsrc(
        static_cast<char *>(g.C) + (static_cast<int64_t>(wm0) * g.N + wn0) * 2, 0, 0x7FFFFFFF, 0x00020000);
    const int rr0 = lane >> 3, cc = (lane & 7) * 8;     // 8 lanes cover a 128-byte row segment, 8 rows per instruction
    const int voff = (rr0 * g.N + cc) * 2;
    char *const wr = slab + fr * PITCH + fh * 8;
    const char *const rd = slab + rr0 * PITCH + cc * 2;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {      // columns 64 ch .. 64 ch + 63 of the wavefront's 128
            __builtin_amdgcn_sched_barrier(0);
            // The two accumulators of this piece pass through an opaque statement that keeps them where
            // the MFMAs left them (accumulation registers): their 32 values are moved to vector registers
            // here, piece by piece, not all 256 at the end of the k loop with everything else still live.
            asm volatile("" : "+a"(acc[i][ch * 2]), "+a"(acc[i][ch * 2 + 1]));
#pragma unroll
            for (int jl = 0; jl < 2; ++jl)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int j = ch * 2 + jl;
                    f32x4 o;
                    if (KIND == 1) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = Mma<KIND>::to_float(acc[i][j][vg * 4 + e]) * g.alpha;
                    } else {
                        const f32x4 c = *reinterpret_cast<const f32x4 *>(csl + j * 32 + vg * 8 + fh * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = Mma<KIND>::to_float(acc[i][j][vg * 4 + e]) * (sa[i] * c[e]);
                    }
                    u32x2 p = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
                    *reinterpret_cast<u32x2 *>(wr + (jl * 32 + vg * 8) * 2) = p;
                }
            lds_wave_fence();
            u32x4 v[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) v[p] = *reinterpret_cast<const u32x4 *>(rd + p * 8 * PITCH);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int row = i * 32 + p * 8;                     // + rr0: this lane's row within the sub-tile
                const int soff = (row * g.N + ch * 64) * 2;         // wave-uniform part of the offset
                const int mm = wm0 + row + rr0, n = wn0 + ch * 64 + cc;
                if ((g.N & 7) == 0) {
                    if (interior || (mm < g.M && n < g.N)) __builtin_amdgcn_raw_buffer_store_b128(v[p], rsC, voff, soff, 0);
                } else if (mm < g.M) {   // rows that are only 8-byte aligned: two halves, the last may be missing
                    const u32x2 lo = {v[p][0], v[p][1]}, hi = {v[p][2], v[p][3]};
                    if (n < g.N) __builtin_amdgcn_raw_buffer_store_b64(lo, rsC, voff, soff, 0);
                    if (n + 4 < g.N) __builtin_amdgcn_raw_buffer_store_b64(hi, rsC, voff + 8, soff, 0);
                }
            }
            lds_wave_fence();
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

constexpr size_t gemm_stream_lds_bytes() { return 2u * 65536u + 4u * kStreamEpiBytes; }

template <int KIND>
__device__ __forceinline__ void gemm_stream_product(const GemmDev &g, const int wg, const int nwg)
{
    constexpr int WM = 4, WN = 4, KCH = 8;
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int GROUP = 4;
    constexpr int NS = KCH / 2;
    constexpr int RPP = 256 / KCH;
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int STAGE = (BM + BN) * KCH;
    constexpr uint32_t STAGE_BYTES = STAGE * 16u;
    static_assert(STAGE_BYTES == 65536u && NS == 4 && PA == 8 && PB == 8, "written for 256 x 256 tiles, 128 B of k per step");
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;

    // ---- this workgroup's tiles: logical tiles first + j + t * jn, t = 0 .. ntiles-1, of its XCD's range ----
    const int nb = g.tiles_m * g.tiles_n;
    const int xcd = wg & 7, j = wg >> 3, jn = nwg >> 3;
    const int per = nb >> 3, rem = nb & 7;
    const int first = xcd * per + (xcd < rem ? xcd : rem);
    const int cnt = per + (xcd < rem ? 1 : 0);
    const int ntiles = j < cnt ? (cnt - 1 - j) / jn + 1 : 0;
    if (ntiles == 0) return;
    const int nk = g.Kb / (KCH * 16);

#define HLQ_TILE_OF(T, M0, N0)                                                                                \
    {                                                                                                         \
        const int logical = first + j + (T) * jn;                                                             \
        const int width = GROUP * g.tiles_n;                                                                  \
        const int group = logical / width;                                                                    \
        const int first_m = group * GROUP;                                                                    \
        const int gsz = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;                        \
        const int within = logical - group * width;                                                           \
        M0 = (first_m + within % gsz) * BM;                                                                   \
        N0 = (within / gsz) * BN;                                                                             \
    }

    // ---- load side: the tile whose operand rows are being fetched, and the next k step to fetch ----
    // Rows past the end of an operand are redirected to the tile's first row (they feed accumulators
    // that are never stored), so the loop needs no row predicate.
    const int lc = tid % KCH, lr = tid / KCH;
    const char *ldA, *ldB;
    uint32_t offa[PA], offb[PB];
    int ldt = 0, ldk = 0;
#define HLQ_SET_LOAD_TILE(T)                                                                                  \
    {                                                                                                         \
        int lm0, ln0;                                                                                         \
        HLQ_TILE_OF(T, lm0, ln0)                                                                              \
        ldA = g.A + static_cast<int64_t>(lm0) * g.Kb;                                            \
        ldB = g.Bm + static_cast<int64_t>(ln0) * g.Kb;                                           \
        _Pragma("unroll") for (int i = 0; i < PA; ++i) {                                                      \
            const int row = lr + RPP * i;                                                                     \
            offa[i] = static_cast<uint32_t>(lm0 + row < g.M ? row : 0) * static_cast<uint32_t>(g.Kb) + lc * 16u; \
        }                                                                                                     \
        _Pragma("unroll") for (int jj = 0; jj < PB; ++jj) {                                                   \
            const int row = lr + RPP * jj;                                                                    \
            offb[jj] = static_cast<uint32_t>(ln0 + row < g.N ? row : 0) * static_cast<uint32_t>(g.Kb) + lc * 16u; \
        }                                                                                                     \
    }
    // after the loads of a step have been issued: the next step, in the next tile when this one is
    // exhausted; past the last tile the last step is fetched again (staged, never multiplied)
#define HLQ_ADVANCE_LOAD()                                                                                    \
    {                                                                                                         \
        if (++ldk == nk) {                                                                                    \
            if (ldt + 1 < ntiles) {                                                                           \
                ++ldt;                                                                                        \
                ldk = 0;                                                                                      \
                HLQ_SET_LOAD_TILE(ldt)                                                                        \
            } else {                                                                                          \
                ldk = nk - 1;                                                                                 \
            }                                                                                                 \
        }                                                                                                     \
    }
    HLQ_SET_LOAD_TILE(0)

    u32x4 ra[PA], rb[PB];
#define HLQ_RSRC(P) __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(P), 0, 0x7FFFFFFF, 0x00020000)
#define HLQ_LOAD_GLOBAL_A()                                                                                   \
    {                                                                                                         \
        const int kuni = ldk * (KCH * 16);                                                                    \
        _Pragma("unroll") for (int i = 0; i < PA; ++i)                                                        \
            ra[i] = __builtin_amdgcn_raw_buffer_load_b128(HLQ_RSRC(ldA), offa[i], kuni, 0);                   \
    }
#define HLQ_LOAD_GLOBAL_B()                                                                                   \
    {                                                                                                         \
        const int kuni = ldk * (KCH * 16);                                                                    \
        _Pragma("unroll") for (int jj = 0; jj < PB; ++jj)                                                     \
            rb[jj] = __builtin_amdgcn_raw_buffer_load_b128(HLQ_RSRC(ldB), offb[jj], kuni, 0);                 \
    }
#define HLQ_LOAD_ONE(W_)                                                                                      \
    {                                                                                                         \
        const int kuni = ldk * (KCH * 16);                                                                    \
        if ((W_) < PA) ra[(W_) < PA ? (W_) : 0] = __builtin_amdgcn_raw_buffer_load_b128(HLQ_RSRC(ldA), offa[(W_) < PA ? (W_) : 0], kuni, 0); \
        else rb[(W_) >= PA ? (W_) - PA : 0] = __builtin_amdgcn_raw_buffer_load_b128(HLQ_RSRC(ldB), offb[(W_) >= PA ? (W_) - PA : 0], kuni, 0); \
    }

    // ---- LDS addressing: as in gemm_body.hpp (one lane register + immediates, stage toggled by xor) ----
    char *const ldsb = reinterpret_cast<char *>(lds);
    const int fr = lane & 31, fh = lane >> 5;
    uint32_t wr_off = lds_chunk<KCH>(lr, lc) * 16u + STAGE_BYTES;
    uint32_t rdA[NS], rdB[NS];
#pragma unroll
    for (int ks = 0; ks < NS; ++ks) {
        rdA[ks] = lds_chunk<KCH>(wave_m * (32 * WM) + fr, ks * 2 + fh) * 16u;
        rdB[ks] = (BM * KCH + lds_chunk<KCH>(wave_n * (32 * WN) + fr, ks * 2 + fh)) * 16u;
    }
#define HLQ_STORE_LDS_A()                                                                                     \
    {                                                                                                         \
        _Pragma("unroll") for (int i = 0; i < PA; ++i)                                                        \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + i * (RPP * KCH * 16)) = ra[i];                         \
    }
#define HLQ_STORE_LDS_B()                                                                                     \
    {                                                                                                         \
        _Pragma("unroll") for (int jj = 0; jj < PB; ++jj)                                                     \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + (BM * KCH * 16) + jj * (RPP * KCH * 16)) = rb[jj];     \
    }
    u32x4 fa[2][WM], fb[2][WN];
#define HLQ_READ_FRAGS(BUF, KS)                                                                               \
    {                                                                                                         \
        fb[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS]);                                        \
        fa[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS]);                                        \
        _Pragma("unroll") for (int jj = 1; jj < WN; ++jj)                                                     \
            fb[BUF][jj] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS] + jj * (32 * KCH * 16));            \
        _Pragma("unroll") for (int i = 1; i < WM; ++i)                                                        \
            fa[BUF][i] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS] + i * (32 * KCH * 16));              \
    }
#define HLQ_READ_ONE(BUF, KS, Q)                                                                              \
    {                                                                                                         \
        if ((Q) == 0) fb[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS]);                          \
        else if ((Q) == 1) fa[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS]);                     \
        else if ((Q) < 1 + WN) fb[BUF][(Q) - 1] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS] + ((Q) - 1) * (32 * KCH * 16)); \
        else fa[BUF][(Q) - WN] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS] + ((Q) - WN) * (32 * KCH * 16)); \
    }
#define HLQ_STORE_ONE(W_)                                                                                     \
    {                                                                                                         \
        if ((W_) < PA)                                                                                        \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + (W_) * (RPP * KCH * 16)) = ra[(W_) < PA ? (W_) : 0];   \
        else                                                                                                  \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + (BM * KCH * 16) + ((W_) - PA) * (RPP * KCH * 16)) =    \
                rb[(W_) >= PA ? (W_) - PA : 0];                                                               \
    }
#define HLQ_TOGGLE_STAGE()                                                                                    \
    {                                                                                                         \
        _Pragma("unroll") for (int ks = 0; ks < NS; ++ks) { rdA[ks] ^= STAGE_BYTES; rdB[ks] ^= STAGE_BYTES; } \
    }
    u32x4 ea[2][WM][2], pb[2];    // packed codes: expanded A operands and first B operand of the coming sub-step
    // the first sub-step's operands of the step the read addresses point at
#define HLQ_FIRST_FRAGS()                                                                                     \
    {                                                                                                         \
        HLQ_READ_FRAGS(0, 0)                                                                                  \
        if constexpr (KIND == 2) {                                                                            \
            _Pragma("unroll") for (int i = 0; i < WM; ++i) Mma<2>::expand(fa[0][i], ea[0][i][0], ea[0][i][1]); \
            Mma<2>::expand(fb[0][0], pb[0], pb[1]);                                                           \
        }                                                                                                     \
    }

    // ---- prologue of the list: steps 0 and 1 of the first tile into the two stages, step 2 into registers ----
    HLQ_LOAD_GLOBAL_A()
    HLQ_LOAD_GLOBAL_B()
    HLQ_ADVANCE_LOAD()
    wr_off ^= STAGE_BYTES;
    HLQ_STORE_LDS_A()
    HLQ_STORE_LDS_B()
    wr_off ^= STAGE_BYTES;
    HLQ_LOAD_GLOBAL_A()
    HLQ_LOAD_GLOBAL_B()
    HLQ_ADVANCE_LOAD()
    HLQ_STORE_LDS_A()
    HLQ_STORE_LDS_B()
    HLQ_LOAD_GLOBAL_A()
    HLQ_LOAD_GLOBAL_B()
    HLQ_ADVANCE_LOAD()
    lds_barrier();

    constexpr int MPS = KIND == 2 ? 2 : 1;
    constexpr bool SPREAD = KIND != 2;

    for (int ct = 0; ct < ntiles; ++ct) {
        int m0, n0;                  // the tile being multiplied
        HLQ_TILE_OF(ct, m0, n0)
        typename Mma<KIND>::acc_t acc[WM][WN];
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int jj = 0; jj < WN; ++jj) acc[i][jj] = Mma<KIND>::zero();

        // One k step: NS sub-steps of WM * WN MFMAs, the fragment reads of the next sub-step under them.
        // With staging (every step but a tile's first): the registers (step + 1) go to the other LDS
        // stage and are refilled from global memory (step + 2, in the next tile near the end of this
        // one), scheduled as in gemm_body.hpp.  Without: both stages are full, nothing moves.
        // Either way one barrier after the third sub-step, and the stage roles swap.
        auto step = [&](auto stg) __attribute__((always_inline)) {
            constexpr bool STG = decltype(stg)::value;
#pragma unroll
            for (int ks = 0; ks < NS; ++ks) {
                const int cur = ks & 1;
                if constexpr (SPREAD) {
                    const int WC = !STG ? 0 : (ks == 0 ? 6 : (ks == 1 ? 6 : (ks == 2 ? 4 : 0)));
                    const int W0 = ks == 0 ? 0 : (ks == 1 ? 6 : 12);
                    if (ks == NS - 1) HLQ_TOGGLE_STAGE()
#pragma unroll
                    for (int q = 0; q < WM * WN; ++q) {
                        if (q < WM + WN) {
                            if (ks < NS - 1) HLQ_READ_ONE(cur ^ 1, ks + 1, q)
                            else HLQ_READ_ONE(cur ^ 1, 0, q)
                        }
                        if ((q & 1) && (q >> 1) < WC) HLQ_STORE_ONE(W0 + (q >> 1))
                        if (!(q & 1) && q >= 2 && ((q - 2) >> 1) < WC) HLQ_LOAD_ONE(W0 + ((q - 2) >> 1))
                    }
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int jj = 0; jj < WN; ++jj) acc[i][jj] = Mma<KIND>::mma(fb[cur][jj], fa[cur][i], acc[i][jj]);
#pragma unroll
                    for (int q = 0; q < WM * WN; ++q) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (q < WM + WN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        if ((q & 1) && (q >> 1) < WC) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                        if (!(q & 1) && q >= 2 && ((q - 2) >> 1) < WC) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    }
                    if (ks == NS - 2) wr_off ^= STAGE_BYTES;
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks == NS - 2) {
                        lds_barrier();
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    continue;
                }
                if (ks < NS - 1) {
                    HLQ_READ_FRAGS(cur ^ 1, ks + 1)
                } else {
                    HLQ_READ_FRAGS(cur ^ 1, 0)
                }
                if constexpr (KIND == 2) {
                    u32x4 eb[2][2];
                    eb[0][0] = pb[0];
                    eb[0][1] = pb[1];
#pragma unroll
                    for (int jj = 0; jj < WN; ++jj) {
                        if (jj + 1 < WN) Mma<2>::expand(fb[cur][jj + 1], eb[(jj + 1) & 1][0], eb[(jj + 1) & 1][1]);
#pragma unroll
                        for (int i = 0; i < WM; ++i) acc[i][jj] = Mma<2>::mma(eb[jj & 1][0], ea[cur][i][0], acc[i][jj]);
#pragma unroll
                        for (int i = 0; i < WM; ++i) acc[i][jj] = Mma<2>::mma(eb[jj & 1][1], ea[cur][i][1], acc[i][jj]);
                    }
#pragma unroll
                    for (int i = 0; i < WM; ++i) Mma<2>::expand(fa[cur ^ 1][i], ea[cur ^ 1][i][0], ea[cur ^ 1][i][1]);
                    Mma<2>::expand(fb[cur ^ 1][0], pb[0], pb[1]);
                    if (ks == NS - 1) {
#pragma unroll
                        for (int i = 0; i < WM; ++i) {
                            asm("" : "+v"(ea[cur ^ 1][i][0]));
                            asm("" : "+v"(ea[cur ^ 1][i][1]));
                        }
                        asm("" : "+v"(pb[0]));
                        asm("" : "+v"(pb[1]));
                    }
                }
                if (STG && ks == 0) {
                    HLQ_STORE_LDS_A()
                    HLQ_LOAD_GLOBAL_A()
                }
                if (STG && ks == 1) {
                    HLQ_STORE_LDS_B()
                    HLQ_LOAD_GLOBAL_B()
                }
                if (ks == 1) wr_off ^= STAGE_BYTES;
                constexpr int VPS = KIND == 2 ? 12 * (WM + WN) / (WM * WN) : 0;
#pragma unroll
                for (int q = 0; q < (WM * WN) / 2; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, MPS, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (WM + WN) / (WM * WN), 0);
                    if (VPS) __builtin_amdgcn_sched_group_barrier(0x002, VPS, 0);
                }
#pragma unroll
                for (int q = 0; q < (WM * WN) / 2; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, MPS, 0);
                    if (VPS) __builtin_amdgcn_sched_group_barrier(0x002, VPS, 0);
                    if (STG && ks < 2) {
                        __builtin_amdgcn_sched_group_barrier(0x200, 2 * PA / (WM * WN), 0);
                        __builtin_amdgcn_sched_group_barrier(0x020, 2 * PA / (WM * WN), 0);
                    }
                }
                if (ks == NS - 2) HLQ_TOGGLE_STAGE()
                __builtin_amdgcn_sched_barrier(0);
                if (ks == NS - 2) {
                    lds_barrier();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };

        HLQ_FIRST_FRAGS()
        step(BoolTag<false>{});
        // Everything issued so far -- the last tile's stores, then this tile's third step -- has had a
        // whole step to complete; waiting for it here costs nothing and leaves the loop below with
        // loads only in flight, which are waited for one by one.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), nothing else
        for (int ck = 1; ck < nk; ++ck) {
            step(BoolTag<true>{});
            HLQ_ADVANCE_LOAD()
        }
        // ---- the tile is complete.  The registers hold the next tile's second step: it goes to the stage
        // the last step has just consumed (every wavefront has passed that step's barrier, which follows
        // its last read of it), next to the next tile's first step in the other stage.
        const bool more = ct + 1 < ntiles;
        if (more) {
            HLQ_STORE_LDS_A()
            HLQ_STORE_LDS_B()
        }
        // The lane and wavefront numbers pass through an opaque statement: nothing the epilogue derives
        // from them can be computed ahead of the loops and held in registers across them, where every
        // register is spoken for.
        int lane_e = lane, wave_e = wave;
        asm volatile("" : "+v"(lane_e), "+v"(wave_e));
        wave_e = __builtin_amdgcn_readfirstlane(wave_e);
        const int wm0 = m0 + (wave_e >> 1) * (32 * WM), wn0 = n0 + (wave_e & 1) * (32 * WN);
        char *area = ldsb + 2 * STAGE_BYTES + wave_e * kStreamEpiBytes;
        const bool interior = (m0 + BM <= g.M) && (n0 + BN <= g.N) && ((g.N & 7) == 0);
        stream_epilogue<KIND>(acc, g, wm0, wn0, lane_e, area, interior);
        if (more) {
            // the next tile's third step, behind the stores
            HLQ_LOAD_GLOBAL_A()
            HLQ_LOAD_GLOBAL_B()
            HLQ_ADVANCE_LOAD()
        }
    }
    // whatever runs next in this workgroup (the other product's list) stages into LDS at once: every
    // wavefront must be done with the operand stages
    lds_barrier();
#undef HLQ_TILE_OF
#undef HLQ_SET_LOAD_TILE
#undef HLQ_ADVANCE_LOAD
#undef HLQ_RSRC
#undef HLQ_LOAD_GLOBAL_A
#undef HLQ_LOAD_GLOBAL_B
#undef HLQ_LOAD_ONE
#undef HLQ_STORE_LDS_A
#undef HLQ_STORE_LDS_B
#undef HLQ_READ_FRAGS
#undef HLQ_READ_ONE
#undef HLQ_STORE_ONE
#undef HLQ_TOGGLE_STAGE
#undef HLQ_FIRST_FRAGS
}

}  // namespace hlq
