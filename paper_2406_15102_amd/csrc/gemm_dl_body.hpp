// Device body of K2 / K4 for 256 x 256 tiles and rows of whole 128-byte steps, with the operands
// streamed from global memory straight into LDS (arXiv 2406.15102, Sec. 6.1: stages 5-6 of the g_x
// list, stage 5 of the g_w list; the same products, tile, MFMA feeding and epilogue as gemm_body.hpp,
// bit for bit the same results).
//
// In gemm_body.hpp an operand chunk travels global -> registers -> LDS.  The ds_write that moves it
// on reads 1 KB of registers per wavefront and holds up the MFMA stream; the round trip through the
// register file also costs power, which on this chip is clock.  `buffer_load ... lds` delivers the
// chunks into LDS without touching the register file.  What it takes to make that pay (measured on
// MI355X with the rocprofv3 counters SQ_VMEM_TA_ADDR_FIFO_FULL, SQ_INST_LEVEL_VMEM, GRBM_GUI_ACTIVE):
//   * a load instruction of a wavefront fetches whole 128-byte lines (8 rows x 128 B) -- with 64-byte
//     steps every line is asked for twice and a load takes 1.7 x as long to land;
//   * loads go out singly between the MFMAs, never in a burst from all four wavefronts (the address
//     queues of the memory pipeline fill up and the wavefront stalls at issue);
//   * LDS is a ring of five 32 KB units -- all 160 KB.  Step kt keeps its A rows in unit 2 kt mod 5 and
//     its Bm rows in the next one, so while step kt is multiplied step kt + 1 is complete or landing
//     in two more units and the fifth takes the A rows of step kt + 2 already: a load has between
//     0.75 and 1.75 steps to land, about what the register-staged pipeline gives it.
// One barrier per step, after the third of its four sub-steps: by then every wavefront has waited
// for its own loads of step kt + 1, and nobody reads step kt from LDS any more (the fragments of
// the last sub-step are in registers), which frees that step's two units for the Bm rows of step
// kt + 2 and, one step later, the A rows of step kt + 3.
#pragma once
#include "gemm_common.hpp"

namespace hlq {

typedef __attribute__((address_space(3))) void lds_void_t;

constexpr size_t kGemmDlLdsBytes = 5u * 256u * 128u;   // the ring; the epilogue's slabs reuse its start

// half of Mma<2>::expand: dwords 2 h and 2 h + 1 of a packed fragment (6 vector instructions)
__device__ __forceinline__ void expand_half(const u32x4 &x, u32x4 &even, u32x4 &odd, int h)
{
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        odd[2 * h + d] = x[2 * h + d] & 0xF0F0F0F0u;
        even[2 * h + d] = (x[2 * h + d] << 4) & 0xF0F0F0F0u;
    }
}

// OUT as in gemm_tile; `bid`: index of the workgroup among those of this product.
// Requires g.Kb % 128 == 0 and tiles of 256 x 256 (g.tiles_m, g.tiles_n counted in such tiles).
template <int KIND, int OUT>
__device__ __forceinline__ void gemm_tile_dl(const GemmDev &g, const int bid)
{
    constexpr int W = 4, BT = 256, GROUP = 4, NS = 4;
    constexpr uint32_t UNIT = BT * 128u;          // one operand's rows of one step: 32 KB
    constexpr uint32_t RING = 5u * UNIT;
    extern __shared__ u32x4 lds[];
    char *const ldsb = reinterpret_cast<char *>(lds);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;

    // ---- workgroup id -> tile, XCD-aware (as in gemm_tile) ----
    int tm, tn;
    {
        const int nb = g.tiles_m * g.tiles_n;
        const int pid = bid % nb;                  // bid / nb is the k split
        const int xcd = pid & 7, idx = pid >> 3;
        const int per = nb >> 3, rem = nb & 7;
        const int logical = xcd * per + (xcd < rem ? xcd : rem) + idx;
        const int width = GROUP * g.tiles_n;
        const int group = logical / width;
        const int first_m = group * GROUP;
        const int gsz = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
        const int within = logical - group * width;
        tm = first_m + within % gsz;
        tn = within / gsz;
    }
    const int m0 = tm * BT, n0 = tn * BT;

    // ---- loads: instruction j of this wavefront fills rows 8 (4 j + wave) .. + 7 of an operand ----
    // 1 KB of LDS in lane order: lane -> row lane / 8 of the block, position lane % 8 of the row, which
    // in the swizzled layout (lds_chunk<8>) holds chunk position ^ (row & 7) ^ (row >> 3 & 1) of that
    // row.  Rows past the end of an operand are redirected to the tile's first row (never stored).
    const char *baseA = g.A + static_cast<int64_t>(m0) * g.Kb;
    const char *baseB = g.Bm + static_cast<int64_t>(n0) * g.Kb;
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(baseA), 0, 0x7FFFFFFF, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(baseB), 0, 0x7FFFFFFF, 0x00020000);
    uint32_t offa[8], offb[8];
    {
        const int rb = lane >> 3, slot = lane & 7;
        const uint32_t c16 = static_cast<uint32_t>(slot ^ rb ^ (wave & 1)) * 16u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = 8 * (4 * j + wave) + rb;
            offa[j] = static_cast<uint32_t>(m0 + row < g.M ? row : 0) * static_cast<uint32_t>(g.Kb) + c16;
            offb[j] = static_cast<uint32_t>(n0 + row < g.N ? row : 0) * static_cast<uint32_t>(g.Kb) + c16;
        }
    }
    const int nk_all = g.Kb / 128;
    const int split = bid / (g.tiles_m * g.tiles_n);
    const int kbeg = static_cast<int>(static_cast<int64_t>(nk_all) * split / g.splits);
    const int nk = static_cast<int>(static_cast<int64_t>(nk_all) * (split + 1) / g.splits) - kbeg;

    // instruction J of operand OP (0 = A, 1 = Bm) of step KT into ring unit UNIT_.  Past the end, steps are
    // clamped to the last one: loaded again into a free unit, never multiplied.
#define HLQD_LOAD_ONE(KT, OP, J, UNIT_)                                                                       \
    {                                                                                                         \
        const int kt_ = (KT) < nk ? (KT) : nk - 1;                                                            \
        const int kuni = (kbeg + kt_) * 128;      /* wave-uniform: lives in an SGPR */                        \
        const uint32_t dst = static_cast<uint32_t>(UNIT_) * UNIT + static_cast<uint32_t>(wave) * 1024u + (J) * 4096u; \
        if ((OP) == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_void_t *)(ldsb + dst), 16, offa[J], kuni, 0, 0); \
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_void_t *)(ldsb + dst), 16, offb[J], kuni, 0, 0); \
    }

    // ---- fragment reads: one per-lane register per (operand, sub-step), holding the ring position ----
    const int fr = lane & 31, fh = lane >> 5;
    uint32_t rdA[NS], rdB[NS];
#pragma unroll
    for (int ks = 0; ks < NS; ++ks) {
        rdA[ks] = lds_chunk<8>(wave_m * 128 + fr, 2 * ks + fh) * 16u;
        rdB[ks] = UNIT + lds_chunk<8>(wave_n * 128 + fr, 2 * ks + fh) * 16u;
    }
    u32x4 fa[2][W], fb[2][W];
    // fragment Q of sub-step KS, in the order the MFMAs consume them: fb[0], fa[0], fb[1..], fa[1..]
#define HLQD_READ_ONE(BUF, KS, Q)                                                                             \
    {                                                                                                         \
        if ((Q) == 0) fb[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS]);                          \
        else if ((Q) == 1) fa[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS]);                     \
        else if ((Q) < 1 + W) fb[BUF][(Q) - 1] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS] + ((Q) - 1) * 4096u); \
        else fa[BUF][(Q) - W] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS] + ((Q) - W) * 4096u);         \
    }
    // packed codes: the A fragments first (they are expanded within the same sub-step), then the Bm ones
#define HLQD_READ_ONE_P(BUF, KS, Q)                                                                           \
    {                                                                                                         \
        if ((Q) < W) fa[BUF][Q] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS] + (Q) * 4096u);             \
        else fb[BUF][(Q) - W] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS] + ((Q) - W) * 4096u);         \
    }
    // the reads of a step are done: the read position of sub-step S2 (A or Bm) moves on two units, mod the ring
#define HLQD_NEXT_UNIT(S2, OP)                                                                                \
    {                                                                                                         \
        uint32_t &r_ = (OP) == 0 ? rdA[S2] : rdB[S2];                                                         \
        const uint32_t a_ = r_ + 2u * UNIT;                                                                   \
        r_ = a_ < a_ - RING ? a_ : a_ - RING;   /* unsigned: a_ - RING wraps when a_ < RING */                \
    }

    typename Mma<KIND>::acc_t acc[W][W];
#pragma unroll
    for (int i = 0; i < W; ++i)
#pragma unroll
        for (int j = 0; j < W; ++j) acc[i][j] = Mma<KIND>::zero();

    // prologue: steps 0 and 1 in flight (units 0, 1 and 2, 3), wait for step 0
#pragma unroll
    for (int j = 0; j < 8; ++j) HLQD_LOAD_ONE(0, 0, j, 0)
#pragma unroll
    for (int j = 0; j < 8; ++j) HLQD_LOAD_ONE(0, 1, j, 1)
#pragma unroll
    for (int j = 0; j < 8; ++j) HLQD_LOAD_ONE(1, 0, j, 2)
#pragma unroll
    for (int j = 0; j < 8; ++j) HLQD_LOAD_ONE(1, 1, j, 3)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070 | (16 & 15) | ((16 >> 4) << 14));   // vmcnt(16): step 0 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int q = 0; q < 2 * W; ++q) HLQD_READ_ONE(0, 0, q)
    u32x4 ea[2][W][2], pb[2];    // packed codes: expanded A operands and first B operand of the coming sub-step
    if constexpr (KIND == 2) {
#pragma unroll
        for (int i = 0; i < W; ++i) Mma<2>::expand(fa[0][i], ea[0][i][0], ea[0][i][1]);
        Mma<2>::expand(fb[0][0], pb[0], pb[1]);
    }

    // Step kt reads units u = 2 kt mod 5 (A) and u + 1 (Bm); step kt + 1 sits in the next two units.
    //   sub-steps 0, 1  the A rows of step kt + 2 go into the one free unit, u + 4 (four loads each)
    //   sub-step 2      the read positions move on; its barrier: every wavefront's loads of step kt + 1
    //                   have landed (all but the 8 youngest have) and nobody reads step kt from LDS any more
    //   sub-step 3      fragments of step kt + 1's first sub-step; the Bm rows of step kt + 2 go into unit u
    // The loop is written slot by slot -- what is to issue around one MFMA (two for the packed codes) --
    // with a scheduling fence after each slot: 16 slots a sub-step, the fragment reads of the next
    // sub-step in the first eight, the loads in the second eight (every other slot in sub-steps 0 and
    // 1, every slot in sub-step 3), a few vector instructions in each.
    int u = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const int ua = u == 0 ? 4 : u - 1;   // (2 kt + 4) mod 5
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            const int cur = ks & 1;
            const int nks = ks < NS - 1 ? ks + 1 : 0;   // the sub-step whose fragments are read now
            if constexpr (KIND != 2) {
#pragma unroll
                for (int q = 0; q < W * W; ++q) {
                    if (q < 2 * W) HLQD_READ_ONE(cur ^ 1, nks, q)
                    if (ks < 2 && q >= 2 * W && (q & 1)) HLQD_LOAD_ONE(kt + 2, 0, 4 * ks + ((q - 2 * W) >> 1), ua)
                    if (ks == 3 && q >= 2 * W) HLQD_LOAD_ONE(kt + 2, 1, q - 2 * W, u)
                    if (ks == 2 && q >= 2 * W) HLQD_NEXT_UNIT((q - 2 * W) >> 1, q & 1)
                    acc[q / W][q % W] = Mma<KIND>::mma(fb[cur][q % W], fa[cur][q / W], acc[q / W][q % W]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // packed codes: every fragment expands to two MFMA operands (12 vector instructions),
                // 32 MFMAs a sub-step, two a slot.  Column j of the accumulators takes slots 4 j .. 4 j + 3
                // (rows 0-1 and 2-3 with the even codes, then with the odd ones).  Half an expansion a
                // slot: the Bm operands of columns 1, 2, 3 in slots 0-5 (column 0's were expanded at the
                // end of the previous sub-step), the next sub-step's four A operands in slots 6-13 --
                // their fragments are read in slots 0-3 -- and its first Bm operand in slots 14-15.
                u32x4 eb[3][2];
                eb[0][0] = pb[0];
                eb[0][1] = pb[1];
#pragma unroll
                for (int q = 0; q < W * W; ++q) {
                    const int j = q >> 2, t = q & 3, half = t >> 1, i0 = 2 * (t & 1);
                    if (q < 2 * W) HLQD_READ_ONE_P(cur ^ 1, nks, q)
                    if (ks < 2 && q >= 2 * W && (q & 1)) HLQD_LOAD_ONE(kt + 2, 0, 4 * ks + ((q - 2 * W) >> 1), ua)
                    if (ks == 3 && q >= 2 * W) HLQD_LOAD_ONE(kt + 2, 1, q - 2 * W, u)
                    if (ks == 2 && q >= 2 * W) HLQD_NEXT_UNIT((q - 2 * W) >> 1, q & 1)
                    if (q < 6) expand_half(fb[cur][1 + (q >> 1)], eb[(1 + (q >> 1)) % 3][0], eb[(1 + (q >> 1)) % 3][1], q & 1);
                    else if (q < 14) expand_half(fa[cur ^ 1][(q - 6) >> 1], ea[cur ^ 1][(q - 6) >> 1][0], ea[cur ^ 1][(q - 6) >> 1][1], q & 1);
                    else expand_half(fb[cur ^ 1][0], pb[0], pb[1], q & 1);
                    acc[i0][j] = Mma<2>::mma(eb[j % 3][half], ea[cur][i0][half], acc[i0][j]);
                    acc[i0 + 1][j] = Mma<2>::mma(eb[j % 3][half], ea[cur][i0 + 1][half], acc[i0 + 1][j]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (ks == NS - 1) {
                    // loop-carried: keep the compiler from moving these expansions to the top of the
                    // next iteration, where they would stand in front of the first MFMA
#pragma unroll
                    for (int i = 0; i < W; ++i) {
                        asm("" : "+v"(ea[cur ^ 1][i][0]));
                        asm("" : "+v"(ea[cur ^ 1][i][1]));
                    }
                    asm("" : "+v"(pb[0]));
                    asm("" : "+v"(pb[1]));
                }
            }
            if (ks == 2) {
                asm volatile("" ::: "memory");   // no memory access of the program may cross the barrier
                __builtin_amdgcn_s_waitcnt(0x0070 | 8);   // vmcnt(8), lgkmcnt(0)
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        u = u + 2 >= 5 ? u - 3 : u + 2;
    }
#undef HLQD_LOAD_ONE
#undef HLQD_READ_ONE
#undef HLQD_NEXT_UNIT
#undef HLQD_READ_ONE_P

    // ---- epilogue (shared with gemm_tile) ----
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);   // every load has landed: LDS is free for staging C
    __syncthreads();
    const int wm0 = m0 + wave_m * 128, wn0 = n0 + wave_n * 128;
    char *slab = ldsb + wave * EpiSlab<W>::BYTES;   // wavefront-private
    const bool interior = (m0 + BT <= g.M) && (n0 + BT <= g.N) && ((g.N & 7) == 0);
    if (OUT == 2) {
        if (interior) store_raw<KIND, W, W, false>(acc, g.acc, g.M, g.N, wm0, wn0, lane);
        else store_raw<KIND, W, W, true>(acc, g.acc, g.M, g.N, wm0, wn0, lane);
    } else if (OUT == 3) {
        int32_t *part = g.partial + static_cast<int64_t>(split) * g.M * g.N;
        if (interior) store_raw<KIND, W, W, false>(acc, part, g.M, g.N, wm0, wn0, lane);
        else store_raw<KIND, W, W, true>(acc, part, g.M, g.N, wm0, wn0, lane);
    } else {
        if (interior) store_scaled<KIND, W, W, OUT == 1, false>(acc, g.C, g.M, g.N, g.sA, g.sB, g.alpha, wm0, wn0, lane, slab);
        else store_scaled<KIND, W, W, OUT == 1, true>(acc, g.C, g.M, g.N, g.sA, g.sB, g.alpha, wm0, wn0, lane, slab);
    }
}

}  // namespace hlq
