// Device body of K2 / K4 for 256 x 256 (or 192 x 256) tiles and rows of whole 128-byte steps, with the operands
// streamed from global memory straight into LDS and multiplied by 16 x 16 MFMAs (arXiv 2406.15102,
// Sec. 6.1: stages 5-6 of the g_x list, stage 5 of the g_w list; the same products, tile, LDS layout
// and bits as gemm_body.hpp).
//
// In gemm_body.hpp an operand chunk travels global -> registers -> LDS.  The ds_write that moves it
// on reads 1 KB of registers per wavefront and holds up the MFMA stream, and the round trip through
// the register file costs power -- which on this chip, power-limited on matrix work, is clock.
// `buffer_load ... lds` delivers the chunks into LDS without touching the register file.  What it
// takes to make that pay (measured on MI355X with the rocprofv3 counters SQ_VMEM_TA_ADDR_FIFO_FULL,
// SQ_INST_LEVEL_VMEM, GRBM_GUI_ACTIVE):
//   * a load instruction of a wavefront fetches whole 128-byte lines (8 rows x 128 B) -- with 64-byte
//     steps every line is asked for twice and a load takes 1.7 x as long to land;
//   * loads go out singly between the MFMAs, never in a burst from all four wavefronts (the address
//     queues of the memory pipeline fill up and the wavefront stalls at issue);
//   * LDS is a ring of five 32 KB units -- all 160 KB.  Step kt keeps its A rows in unit 2 kt mod 5 and
//     its Bm rows in the next one, so while step kt is multiplied step kt + 1 is complete or landing
//     in two more units and the fifth takes the A rows of step kt + 2 already: a load has between
//     0.75 and 1.5 steps to land, about what the register-staged pipeline gives it.
// One barrier per step, before its last sub-step: by then every wavefront has waited for its own
// loads of step kt + 1, and nobody reads step kt from LDS any more (the fragments of the last
// sub-step are in registers), which frees that step's two units for the Bm rows of step kt + 2 and,
// one step later, the A rows of step kt + 3.
//
// MFMA shape: 16 x 16 x 32 (bf16) / 16 x 16 x 64 (int8), 8 x 8 accumulators of four registers per
// wavefront.  A register-resident probe sustains 5-10 % more on these shapes than on the 32 x 32 ones
// at the chip's power limit, and this loop built around them measured 8 % (long reductions) to 4 %
// faster than the same loop on 32 x 32 MFMAs, with the same bits.  Both operands of an MFMA are read as
// 16 rows x 64 B (lane -> row lane % 16, 16-byte chunk lane / 16), one ds_read_b128 each; packed 4-bit
// codes are read as 16 rows x 32 B (8 bytes a lane) and widened to one such operand in registers.
//
// A second tile shape, 192 rows x 256 columns (6 x 8 accumulators per wavefront, three quarters of the
// work), serves the last rows of a product whose 256-row tiles would leave most compute units idle in
// their last round: 11008 x 4096 is 688 tiles of 256 x 256, 2.69 rounds on 256 compute units; with the
// last 2816 rows in 192-row tiles it is 512 + 240 tiles, two rounds and one of three-quarter tiles.
#pragma once
#include "gemm_common.hpp"

namespace hlq {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef float v4f_t __attribute__((ext_vector_type(4)));

constexpr size_t kGemmDlLdsBytes = 5u * 256u * 128u;   // the ring; the epilogue's slabs reuse its start

// 16 x 16 MFMAs.  The MFMA's A operand is fed from Bm and its B operand from A, which leaves a lane with
// C[m][n .. n + 3], m = 16 i + lane % 16, n = 16 j + 4 (lane / 16), of accumulator (i, j).
// Written out as instructions with the accumulator tied to the destination: through the builtins the
// compiler is free to give an MFMA of this size a destination other than its addend, and with all 256
// accumulator registers in use it then moves dozens of accumulators around at the top of every k step.
// What the compiler's hazard handling no longer sees is kept apart by construction: an accumulator is
// touched by one MFMA in 64, operands written by vector instructions (the widened codes) are written a
// sub-step before they are multiplied, and the epilogue waits out the last MFMAs before it reads.
template <int KIND> struct Mma16;
template <> struct Mma16<0> {
    typedef v4i acc_t;
    static __device__ __forceinline__ acc_t zero() { return acc_t{0, 0, 0, 0}; }
    static __device__ __forceinline__ void mma(const u32x4 &x, const u32x4 &y, acc_t &c)
    {
        asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(c) : "v"(x), "v"(y));
    }
};
template <> struct Mma16<1> {
    typedef v4f_t acc_t;
    static __device__ __forceinline__ acc_t zero() { return acc_t{0.0f, 0.0f, 0.0f, 0.0f}; }
    static __device__ __forceinline__ void mma(const u32x4 &x, const u32x4 &y, acc_t &c)
    {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(x), "v"(y));
    }
};
// packed 4-bit codes: 8 bytes (16 codes) widen to one int8 operand, the even codes in its low half and the
// odd ones in its high half, each moved to the high nibble of its byte (16 x the code, sign included: see
// Mma<2>).  Both operands of a product widen the same way, so which code meets which lane does not matter.
template <> struct Mma16<2> : Mma16<0> {
    // part 0: the odd codes (2 instructions), parts 1, 2: one dword of the even codes each (2 instructions)
    static __device__ __forceinline__ void expand_part(const u32x2 &x, u32x4 &o, int part)
    {
        if (part == 0) {
            o[2] = x[0] & 0xF0F0F0F0u;
            o[3] = x[1] & 0xF0F0F0F0u;
        } else {
            o[part - 1] = (x[part - 1] << 4) & 0xF0F0F0F0u;
        }
    }
};

// raw 32-bit accumulators of the 16 x 16 layout (parity export, split-k partials): direct 16-byte stores
template <int KIND, int NBM, bool GUARD>
__device__ __forceinline__ void store_raw16(typename Mma16<KIND>::acc_t (&acc)[NBM][8], int32_t *out, int M, int N, int wm0,
                                            int wn0, int lane)
{
    const int fr = lane & 15, fq = lane >> 4;
#pragma unroll
    for (int i = 0; i < NBM; ++i) {
        const int m = wm0 + i * 16 + fr;
        int32_t *row = out + static_cast<int64_t>(m) * N + wn0 + fq * 4;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (!GUARD || (m < M && wn0 + j * 16 + fq * 4 < N)) {
                const auto e0 = acc[i][j][0], e1 = acc[i][j][1], e2 = acc[i][j][2], e3 = acc[i][j][3];
                v4i raw = {Mma<KIND>::raw(e0), Mma<KIND>::raw(e1), Mma<KIND>::raw(e2), Mma<KIND>::raw(e3)};
                *reinterpret_cast<v4i *>(row + j * 16) = raw;
            }
        }
    }
}

// C = alpha * sA[m] * sB[n] * acc for the 16 x 16 layout, the arithmetic of store_scaled value for value;
// staged per 16-row group through LDS so that global stores are 16-byte, row-contiguous pieces.
template <int KIND, int NBM, bool F32, bool GUARD>
__device__ __forceinline__ void store_scaled16(typename Mma16<KIND>::acc_t (&acc)[NBM][8], void *Cout, int M, int N,
                                               const float *sA, const float *sB, float alpha, int wm0, int wn0, int lane,
                                               char *slab)
{
    constexpr int PITCH = 128 * (F32 ? 4 : 2) + 16;
    constexpr int EPL = F32 ? 4 : 8;       // elements per 16-byte piece
    constexpr int LPR = 128 / EPL;         // lanes per row
    constexpr int RPI = 64 / LPR;          // rows per store instruction
    const int fr = lane & 15, fq = lane >> 4;
    f32x4 cs[8];
    if (KIND == 1) {
        // unused
    } else if (sB) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            int n = wn0 + j * 16 + fq * 4;
            if (GUARD) n = n < N ? n : 0;
            cs[j] = *reinterpret_cast<const f32x4 *>(sB + n) * alpha;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) cs[j] = f32x4{alpha, alpha, alpha, alpha};
    }
    float sa[NBM];
#pragma unroll
    for (int i = 0; i < NBM; ++i) {
        int m = wm0 + i * 16 + fr;
        if (GUARD) m = m < M ? m : 0;
        sa[i] = sA ? sA[m] : 1.0f;
    }
    const int rr0 = lane / LPR, cc = (lane % LPR) * EPL;
    char *wr = slab + fr * PITCH + fq * 4 * (F32 ? 4 : 2);
    const char *rd = slab + rr0 * PITCH + cc * (F32 ? 4 : 2);
#pragma unroll
    for (int i = 0; i < NBM; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            f32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (KIND == 1) o[e] = Mma<KIND>::to_float(acc[i][j][e]) * alpha;   // no scales on the bf16 product
                else o[e] = Mma<KIND>::to_float(acc[i][j][e]) * (sa[i] * cs[j][e]);
            }
            if (F32) {
                *reinterpret_cast<f32x4 *>(wr + (j * 16) * 4) = o;
            } else {
                u32x2 p = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
                *reinterpret_cast<u32x2 *>(wr + (j * 16) * 2) = p;
            }
        }
        lds_wave_fence();
        u32x4 v[16 / RPI];
#pragma unroll
        for (int p = 0; p < 16 / RPI; ++p) v[p] = *reinterpret_cast<const u32x4 *>(rd + p * RPI * PITCH);
        const int mbase = wm0 + i * 16 + rr0;
        char *dst = static_cast<char *>(Cout) + (static_cast<int64_t>(mbase) * N + wn0 + cc) * (F32 ? 4 : 2);
        const int64_t step = static_cast<int64_t>(RPI) * N * (F32 ? 4 : 2);
#pragma unroll
        for (int p = 0; p < 16 / RPI; ++p) {
            if (!GUARD) {
                *reinterpret_cast<u32x4 *>(dst + p * step) = v[p];
            } else {
                const int m = mbase + p * RPI, n = wn0 + cc;
                if (m < M) {
                    if (F32 || (N & 7) == 0) {
                        if (n < N) *reinterpret_cast<u32x4 *>(dst + p * step) = v[p];
                    } else {   // bf16 rows that are only 8-byte aligned: two halves, the last may be missing
                        const u32x2 lo = {v[p][0], v[p][1]}, hi = {v[p][2], v[p][3]};
                        if (n < N) *reinterpret_cast<u32x2 *>(dst + p * step) = lo;
                        if (n + 4 < N) *reinterpret_cast<u32x2 *>(dst + p * step + 8) = hi;
                    }
                }
            }
        }
        lds_wave_fence();
    }
}

// OUT as in gemm_tile; `bid`: index of the workgroup among those of this product.
// Requires g.Kb % 128 == 0 and tiles of 32 NBM rows x 256 columns, NBM = 8 or 6 (g.tiles_m, g.tiles_n counted
// in such tiles; the 192-row tile is not written for packed codes).
template <int KIND, int NBM, int OUT>
__device__ __forceinline__ void gemm_tile_dl(const GemmDev &g, const int bid)
{
    constexpr int BT = 256, BTM = 32 * NBM, GROUP = 4, NB = 8;
    constexpr bool PACKED = KIND == 2;
    static_assert(NBM == 8 || (NBM == 6 && !PACKED), "tiles of 256 x 256, or 192 x 256 for byte and bf16 operands");
    constexpr int NS = PACKED ? 4 : 2;            // sub-steps per step: 32 B of packed codes, 64 B otherwise
    constexpr int SLOTS = NBM * NB;               // MFMAs of a sub-step, one per accumulator
    constexpr int NR = NBM + NB;                  // fragments of a sub-step
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
    const int m0 = tm * BTM, n0 = tn * BT;

    // ---- loads: instruction j of this wavefront fills rows 8 (4 j + wave) .. + 7 of an operand ----
    // (NBM instructions for the A rows, 8 for the Bm rows)
    // 1 KB of LDS in lane order: lane -> row lane / 8 of the block, position lane % 8 of the row, which
    // in the swizzled layout (lds_chunk<8>) holds chunk position ^ (row & 7) ^ (row >> 3 & 1) of that
    // row.  Rows past the end of an operand are redirected to the tile's first row (never stored).
    const char *baseA = g.A + static_cast<int64_t>(m0) * g.Kb;
    const char *baseB = g.Bm + static_cast<int64_t>(n0) * g.Kb;
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(baseA), 0, 0x7FFFFFFF, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(baseB), 0, 0x7FFFFFFF, 0x00020000);
    uint32_t offa[NBM], offb[8];
    {
        const int rb = lane >> 3, slot = lane & 7;
        const uint32_t c16 = static_cast<uint32_t>(slot ^ rb ^ (wave & 1)) * 16u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = 8 * (4 * j + wave) + rb;
            if (j < NBM) offa[j < NBM ? j : 0] = static_cast<uint32_t>(m0 + row < g.M ? row : 0) * static_cast<uint32_t>(g.Kb) + c16;
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
    // lane -> row lane % 16 of a 16-row block; bytes 16 (lane / 16) .. + 15 of the sub-step's 64 B, or, for
    // packed codes, bytes 8 (lane / 16) .. + 7 of its 32 B.  Block i of an operand is 2 KB further.
    const int fr = lane & 15, fq = lane >> 4;
    uint32_t rdA[NS], rdB[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int chunk = PACKED ? 2 * s + (fq >> 1) : 4 * s + fq;
        const uint32_t half = PACKED ? static_cast<uint32_t>(fq & 1) * 8u : 0u;
        rdA[s] = lds_chunk<8>(wave_m * (16 * NBM) + fr, chunk) * 16u + half;
        rdB[s] = UNIT + lds_chunk<8>(wave_n * 128 + fr, chunk) * 16u + half;
    }
    // the reads of a step are done: the read position of sub-step S2 (A or Bm) moves on two units, mod the ring
#define HLQD_NEXT_UNIT(S2, OP)                                                                                \
    {                                                                                                         \
        uint32_t &r_ = (OP) == 0 ? rdA[S2] : rdB[S2];                                                         \
        const uint32_t a_ = r_ + 2u * UNIT;                                                                   \
        r_ = a_ < a_ - RING ? a_ : a_ - RING;   /* unsigned: a_ - RING wraps when a_ < RING */                \
    }
    // MFMA operands, double-buffered by sub-step: fb[.][j] the Bm blocks, fa[.][i] the A blocks.  For packed
    // codes they hold the widened operands, and pk the 8-byte pieces between their read and their widening.
    u32x4 fa[2][NBM], fb[2][NB];
    u32x2 pk[NR];
    // fragment Q of sub-step S (0-7: Bm blocks -- the first row of MFMAs takes them all --, 8-15: A blocks)
#define HLQD_READ_ONE(BUF, S, Q)                                                                              \
    {                                                                                                         \
        if constexpr (PACKED) {                                                                               \
            if ((Q) < NB) pk[Q] = *reinterpret_cast<const u32x2 *>(ldsb + rdB[S] + (Q) * 2048u);              \
            else pk[Q] = *reinterpret_cast<const u32x2 *>(ldsb + rdA[S] + ((Q) - NB) * 2048u);                \
        } else {                                                                                              \
            if ((Q) < NB) fb[BUF][Q] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[S] + (Q) * 2048u);         \
            else fa[BUF][(Q) - NB] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[S] + ((Q) - NB) * 2048u);    \
        }                                                                                                     \
    }
    // packed codes: part P (0-2) of the widening of fragment Q into the operands of buffer BUF
#define HLQD_EXPAND(BUF, Q, P)                                                                                \
    {                                                                                                         \
        if ((Q) < NB) Mma16<2>::expand_part(pk[Q], fb[BUF][Q], P);                                            \
        else Mma16<2>::expand_part(pk[Q], fa[BUF][(Q) - NB], P);                                              \
    }

    typename Mma16<KIND>::acc_t acc[NBM][NB];
#pragma unroll
    for (int i = 0; i < NBM; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = Mma16<KIND>::zero();

    // prologue: steps 0 and 1 in flight (units 0, 1 and 2, 3), wait for step 0
#pragma unroll
    for (int j = 0; j < NBM; ++j) HLQD_LOAD_ONE(0, 0, j, 0)
#pragma unroll
    for (int j = 0; j < 8; ++j) HLQD_LOAD_ONE(0, 1, j, 1)
#pragma unroll
    for (int j = 0; j < NBM; ++j) HLQD_LOAD_ONE(1, 0, j, 2)
#pragma unroll
    for (int j = 0; j < 8; ++j) HLQD_LOAD_ONE(1, 1, j, 3)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070 | (NR & 15) | ((NR >> 4) << 14));   // vmcnt(NR): step 0 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int q = 0; q < NR; ++q) HLQD_READ_ONE(0, 0, q)
    if constexpr (PACKED) {
#pragma unroll
        for (int q = 0; q < NR; ++q)
#pragma unroll
            for (int p = 0; p < 3; ++p) HLQD_EXPAND(0, q, p)
        // an MFMA may not read a register within two instructions of the vector instruction that wrote it;
        // inside the loop a sub-step lies between the two, here nothing does
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            asm volatile("" ::"v"(fb[0][q]));   // computed before this point ...
            asm volatile("" ::"v"(fa[0][q]));
        }
        asm volatile("s_nop 1");                // ... and two instructions ahead of the first MFMA
    }

    // Step kt reads units u = 2 kt mod 5 (A) and u + 1 (Bm); step kt + 1 sits in the next two units.
    // Every sub-step is 64 MFMAs -- accumulator (q / 8, q % 8) in slot q -- and reads the 16 fragments of
    // the next sub-step in the even slots of its first half (packed codes: see below).  The loop is written
    // slot by slot, what is to issue around one MFMA, with a scheduling fence after each slot, so the issue
    // order is the source order.
    //   all but the last sub-step   the A rows of step kt + 2 go into the one free unit, u + 4, evenly spread
    //   last but one                the read positions move on; its barrier: every wavefront's loads of
    //                               step kt + 1 have landed (all but the 8 youngest have) and nobody reads
    //                               step kt from LDS any more
    //   last                        fragments of step kt + 1's first sub-step; the Bm rows of step kt + 2
    //                               go into unit u, one load every fourth slot of its first half
    int u = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const int ua = u == 0 ? 4 : u - 1;   // (2 kt + 4) mod 5
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int cur = s & 1;
            const int ns = s < NS - 1 ? s + 1 : 0;       // the sub-step whose fragments are read now
            if constexpr (!PACKED) {
                constexpr int APER = SLOTS * (NS - 1) / NBM;   // slots between two loads of A rows
#pragma unroll
                for (int q = 0; q < SLOTS; ++q) {
                    if (q < 2 * NR && !(q & 1)) HLQD_READ_ONE(cur ^ 1, ns, q >> 1)
                    if (s < NS - 1 && (s * SLOTS + q) % APER == APER - 3) HLQD_LOAD_ONE(kt + 2, 0, (s * SLOTS + q) / APER, ua)
                    if (s == NS - 1 && q < 4 * NB && (q & 3) == 1) HLQD_LOAD_ONE(kt + 2, 1, q >> 2, u)
                    if (s == NS - 2 && q >= 4 * NB && q < 4 * NB + 2 * NS) HLQD_NEXT_UNIT((q - 4 * NB) >> 1, q & 1)
                    Mma16<KIND>::mma(fb[cur][q % NB], fa[cur][q / NB], acc[q / NB][q % NB]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // packed codes: a slot has room for the MFMA and 12 more cycles of issue -- two fragment reads,
                // or one part of a widening (two instructions), or a load.  Slots 0-7 read the 16 fragments,
                // slots 12, 18, ..., 54 are kept for the loads (three of the A rows in sub-steps 0 and 1, two in
                // sub-step 2, the eight of the Bm rows in sub-step 3; read positions move on in those that stay
                // free: the one just used, and in sub-step 0 also the one that sub-step 3 will use), and the 48
                // parts of the widening take the other slots from 8 on.
#pragma unroll
                for (int q = 0; q < SLOTS; ++q) {
                    const bool lslot = q >= 12 && q <= 54 && (q - 12) % 6 == 0;
                    const int li = (q - 12) / 6;                       // which of the eight load slots
                    if (q < NB) {
                        HLQD_READ_ONE(cur ^ 1, ns, 2 * q)
                        HLQD_READ_ONE(cur ^ 1, ns, 2 * q + 1)
                    }
                    if (lslot) {
                        if (s < 2 && li % 3 == 1) HLQD_LOAD_ONE(kt + 2, 0, 3 * s + li / 3, ua)
                        if (s == 2 && (li == 1 || li == 4)) HLQD_LOAD_ONE(kt + 2, 0, 6 + li / 3, ua)
                        if (s == 3) HLQD_LOAD_ONE(kt + 2, 1, li, u)
                        if (s < 3 && (li == 3 || li == 6)) HLQD_NEXT_UNIT(ns, li == 6)
                        if (s == 0 && (li == 0 || li == 2)) HLQD_NEXT_UNIT(0, li == 2)
                    }
                    if (q >= 8 && !lslot) {
                        const int e = q - 8 - (q > 12 ? (q < 54 ? (q - 12 + 5) / 6 : 8) : 0);   // rank among the widening slots
                        HLQD_EXPAND(cur ^ 1, e / 3, e % 3)
                    }
                    Mma16<KIND>::mma(fb[cur][q % NB], fa[cur][q / NB], acc[q / NB][q % NB]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (s == NS - 2) {
                asm volatile("" ::: "memory");   // no memory access of the program may cross the barrier
                __builtin_amdgcn_s_waitcnt(0x0070 | NBM);   // vmcnt(NBM): all but the A rows of step kt + 2; lgkmcnt(0)
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
#undef HLQD_EXPAND

    // ---- epilogue ----
    // the last MFMAs have written their accumulators (the compiler does not know that the statements
    // above are MFMAs and would not keep the reads below far enough from them by itself)
    asm volatile("s_nop 15\n\ts_nop 15");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);   // every load has landed: LDS is free for staging C
    __syncthreads();
    const int wm0 = m0 + wave_m * (16 * NBM), wn0 = n0 + wave_n * 128;
    char *slab = ldsb + wave * (16 * (128 * 4 + 16));   // wavefront-private, one 16-row group
    const bool interior = (m0 + BTM <= g.M) && (n0 + BT <= g.N) && ((g.N & 7) == 0);
    if (OUT == 2) {
        if (interior) store_raw16<KIND, NBM, false>(acc, g.acc, g.M, g.N, wm0, wn0, lane);
        else store_raw16<KIND, NBM, true>(acc, g.acc, g.M, g.N, wm0, wn0, lane);
    } else if (OUT == 3) {
        int32_t *part = g.partial + static_cast<int64_t>(split) * g.M * g.N;
        if (interior) store_raw16<KIND, NBM, false>(acc, part, g.M, g.N, wm0, wn0, lane);
        else store_raw16<KIND, NBM, true>(acc, part, g.M, g.N, wm0, wn0, lane);
    } else {
        if (interior) store_scaled16<KIND, NBM, OUT == 1, false>(acc, g.C, g.M, g.N, g.sA, g.sB, g.alpha, wm0, wn0, lane, slab);
        else store_scaled16<KIND, NBM, OUT == 1, true>(acc, g.C, g.M, g.N, g.sA, g.sB, g.alpha, wm0, wn0, lane, slab);
    }
}

}  // namespace hlq
