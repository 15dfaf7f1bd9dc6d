// K2 | K4 in one launch.  The two products of a backward pass (arXiv 2406.15102, Sec. 6.1: stage 5
// of the g_x list and stage 5 of the g_w list) do not depend on each other, and for all but the
// largest layers neither fills the chip by itself: 150 tiles of 256 x 256 at the ViT MLP, a
// handful at a ResNet layer, against 256 compute units.  Launched together, the tiles of one fill
// the compute units the other leaves idle, the tail of one overlaps the start of the other, and
// one launch latency goes away.  A workgroup runs the tile body of gemm_body.hpp of whichever
// product its index falls in (first the tiles of the product with the longer tiles, padded to a
// multiple of 8 so that the other product's tiles keep their XCD assignment, then the other's).  The tile sizes and
// the k split of the g_w product are planned for the pair, not for each product alone.
//
// One translation unit per pair of operand kinds (k_gemm_pair_*.hip instantiate launch_pair_kinds
// below: 100 kernels each -- two tile sizes and whole or ragged k steps per product, the 256-tile also with
// its operands loaded straight into LDS, bf16 or fp32
// output, direct output or split-k partials for the g_w product); k_gemm_pair.hip plans and dispatches.
#pragma once
#include "gemm_body.hpp"
#include "gemm_dl_body.hpp"
#include "gemm_plan.hpp"

namespace hlq {

// MODE: 0 = rows of whole 128-byte steps, 1 = a ragged last step, 2 = whole steps loaded straight into
// LDS (gemm_dl_body.hpp; 256-tiles only)
template <int KIND_, int W_, int MODE_, int OUT_> struct TileCfg {
    static constexpr int KIND = KIND_, W = W_, OUT = OUT_, MODE = MODE_;
    static constexpr size_t LDS = MODE_ == 2 ? kGemmDlLdsBytes : gemm_lds_bytes(W_, W_, 8);
    static_assert(MODE_ != 2 || W_ == 4, "the direct-to-LDS body is written for 256 x 256 tiles");
};

template <class C>
__device__ __forceinline__ void pair_tile(const GemmDev &g, int idx)
{
    if constexpr (C::MODE == 2) gemm_tile_dl<C::KIND, 8, C::OUT>(g, idx);
    else gemm_tile<C::KIND, C::W, C::W, 8, C::MODE == 1, C::OUT>(g, idx);
}
// whether a product of this configuration may hand its last rows to 192-row tiles (gemm_dl_body.hpp)
template <class C> constexpr bool pair_has_tail() { return C::MODE == 2 && C::KIND != 2 && (C::OUT == 0 || C::OUT == 1); }
template <class C>
__device__ __forceinline__ void pair_tail_tile(const GemmDev &g, int idx)
{
    if constexpr (pair_has_tail<C>()) gemm_tile_dl<C::KIND, 6, C::OUT>(g, idx);
}

// n0 workgroups of the product that goes first (padded to n0_pad), then the other's; b_first: the
// g_w product goes first (the plan puts the product with the longer tiles first).  gbt: the last rows
// of the g_w product in 192-row tiles (gbt.tiles_m = 0: none), behind its nb_main other workgroups.
template <class CA, class CB>
__global__ __launch_bounds__(256) void k_gemm_pair(GemmDev ga, GemmDev gb, GemmDev gbt, int nb_main, int n0, int n0_pad,
                                                   int b_first)
{
    const int b = static_cast<int>(blockIdx.x);
    const bool in_first = b < n0_pad;
    if (in_first && b >= n0) return;                    // padding
    const int idx = in_first ? b : b - n0_pad;
    if (in_first != (b_first != 0)) {
        pair_tile<CA>(ga, idx);
        return;
    }
    if (pair_has_tail<CB>() && idx >= nb_main) {
        pair_tail_tile<CB>(gbt, idx - nb_main);
        return;
    }
    pair_tile<CB>(gb, idx);
}

template <class CA, class CB>
static hipError_t launch_pair_tt(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt_in, bool b_first, hipStream_t st)
{
    const GemmDev &gbt = gbt_in;
    if (!pair_has_tail<CB>() && gbt.tiles_m != 0) return hipErrorInvalidValue;   // rows cut off for a kernel that has no tail part
    constexpr size_t lds_bytes = CA::LDS > CB::LDS ? CA::LDS : CB::LDS;
    static bool attr_set = false;     // idempotent; racing callers set the same value
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_pair<CA, CB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nA = ga.tiles_m * ga.tiles_n * ga.splits, nb_main = gb.tiles_m * gb.tiles_n * gb.splits;
    const int nB = nb_main + gbt.tiles_m * gbt.tiles_n;
    const int n0 = b_first ? nB : nA, n1 = b_first ? nA : nB;
    const int n0_pad = (n0 + 7) & ~7;
    hipLaunchKernelGGL((k_gemm_pair<CA, CB>), dim3(n0_pad + n1), dim3(256), lds_bytes, st, ga, gb, gbt, nb_main, n0, n0_pad,
                       b_first ? 1 : 0);
    return hipGetLastError();
}

// the g_w product writes the dtype the g_x product writes (CA::OUT), or its split-k partials
template <class CA, int KB, int WB, int MODEB>
static hipError_t launch_pair_b(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, int outB, bool b_first,
                                hipStream_t st)
{
    if (outB == 3) return launch_pair_tt<CA, TileCfg<KB, WB, MODEB, 3>>(ga, gb, gbt, b_first, st);
    return launch_pair_tt<CA, TileCfg<KB, WB, MODEB, CA::OUT>>(ga, gb, gbt, b_first, st);
}

template <class CA, int KB>
static hipError_t launch_pair_a(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigB, int modeB, int outB,
                                bool b_first, hipStream_t st)
{
    if (bigB) {
        if (modeB == 2) return launch_pair_b<CA, KB, 4, 2>(ga, gb, gbt, outB, b_first, st);
        return modeB ? launch_pair_b<CA, KB, 4, 1>(ga, gb, gbt, outB, b_first, st) : launch_pair_b<CA, KB, 4, 0>(ga, gb, gbt, outB, b_first, st);
    }
    return modeB ? launch_pair_b<CA, KB, 2, 1>(ga, gb, gbt, outB, b_first, st) : launch_pair_b<CA, KB, 2, 0>(ga, gb, gbt, outB, b_first, st);
}

template <int KA, int KB, int WA, int MODEA>
static hipError_t launch_pair_o(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool f32, bool bigB, int modeB,
                                int outB, bool b_first, hipStream_t st)
{
    return f32 ? launch_pair_a<TileCfg<KA, WA, MODEA, 1>, KB>(ga, gb, gbt, bigB, modeB, outB, b_first, st)
               : launch_pair_a<TileCfg<KA, WA, MODEA, 0>, KB>(ga, gb, gbt, bigB, modeB, outB, b_first, st);
}

// every kernel of one pair of kinds; the plan comes from the caller
template <int KA, int KB>
static hipError_t launch_pair_kinds(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigA, bool f32, bool bigB,
                                    int outB, bool b_first, hipStream_t st)
{
    const int modeA = ga.Kb % 128 != 0 ? 1 : (bigA && gemm_dl_ok(ga.Kb, ga.splits) ? 2 : 0);
    const int modeB = gb.Kb % 128 != 0 ? 1 : (bigB && gemm_dl_ok(gb.Kb, gb.splits) ? 2 : 0);
    if (bigA) {
        if (modeA == 2) return launch_pair_o<KA, KB, 4, 2>(ga, gb, gbt, f32, bigB, modeB, outB, b_first, st);
        return modeA ? launch_pair_o<KA, KB, 4, 1>(ga, gb, gbt, f32, bigB, modeB, outB, b_first, st)
                     : launch_pair_o<KA, KB, 4, 0>(ga, gb, gbt, f32, bigB, modeB, outB, b_first, st);
    }
    return modeA ? launch_pair_o<KA, KB, 2, 1>(ga, gb, gbt, f32, bigB, modeB, outB, b_first, st)
                 : launch_pair_o<KA, KB, 2, 0>(ga, gb, gbt, f32, bigB, modeB, outB, b_first, st);
}

}  // namespace hlq
