// Device body of K2 / K4 -- the two matrix products of the HLQ backward pass (arXiv 2406.15102, Sec. 6.1):
//   K2  stage 5-6 of the g_x list: int8 x int8 -> int32 product of the 4-bit codes (exact), then
//       dequantisation by the two per-row scales and 1/B            (v_mfma_i32_32x32x32_i8)
//   K4  stage 5 of the g_w list: bf16 product over the compressed token axis, fp32 accumulation,
//       scaled by 1/B                                               (v_mfma_f32_32x32x16_bf16)
// Both are "NT" products C[m,n] = sum_k A[m,k] Bm[n,k] with the reduction axis contiguous in both
// operands, and both MFMA shapes consume 16 B per lane and operand for a 32-byte slice of k, so one
// kernel template written in bytes serves the two.
//
// Tiling: a workgroup of 4 wavefronts (2 x 2), one per SIMD, owns a (64*WM) x (64*WN) tile of C;
// each wavefront a (32*WM) x (32*WN) sub-tile held as WM x WN MFMA accumulators (AGPRs).  That is
// the shape with the least LDS traffic per MFMA, which is what bounds a 256 x 256 tile.
//
// Pipeline: k advances KCH*16 bytes per step through two LDS stages.  Within a step the wavefront
// runs KCH/2 sub-steps of WM*WN MFMAs; the operand fragments of sub-step s+1 are read from LDS
// while the MFMAs of sub-step s execute, global loads run two steps ahead of the MFMAs in
// registers, and the single workgroup barrier of a step waits on LDS traffic only, so neither
// LDS nor global latency is exposed to the one wavefront a SIMD has.
// LDS rows hold KCH 16-byte chunks; the chunk index is xor-swizzled with the row so that both
// the fragment reads (32 consecutive rows, one chunk) and the staging writes spread over all banks.
// The MFMA's A operand is fed from Bm and its B operand from A, which leaves each lane with four
// consecutive n for one m.  The epilogue scales the accumulators, stages each 32-row slab of the
// wavefront's sub-tile in LDS and writes C in full 16-byte, row-contiguous pieces.
// Workgroup ids are remapped so that each XCD (ids congruent mod 8) works on a compact patch of
// tiles and re-uses operand rows in its own L2.
#pragma once
#include "gemm_common.hpp"

namespace hlq {

// OUT: 0 = C in bf16, 1 = C in fp32, 2 = raw int32 accumulators (parity export),
//      3 = raw 32-bit partial accumulators of this workgroup's k range (split-K)
// `bid`: index of the workgroup among those of this product (tile and k split are derived from it).
template <int KIND, int WM, int WN, int KCH, bool TAIL, int OUT>
__device__ __forceinline__ void gemm_tile(const GemmDev &g, const int bid)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int GROUP = 4;
    constexpr int NS = KCH / 2;                 // MFMA sub-steps (32 B of k) per step
    constexpr int RPP = 256 / KCH;              // tile rows staged per pass of the workgroup
    constexpr int PA = BM / RPP, PB = BN / RPP; // passes per operand
    constexpr int STAGE = (BM + BN) * KCH;      // 16-B chunks per LDS stage
    extern __shared__ u32x4 lds[];              // 2 * STAGE chunks

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;

    // ---- workgroup id -> tile, XCD-aware ----
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
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- staging assignment: thread -> (row, chunk); addresses = uniform tile base + 32-bit offset ----
    // Rows past the end of an operand are redirected to the tile's first row: they only feed
    // accumulators that the epilogue never stores, so the main loop needs no row predicate.
    const int lc = tid % KCH;     // 16-B chunk within the k step
    const int lr = tid / KCH;     // row 0..RPP-1 (+RPP i)
    const char *baseA = g.A + static_cast<int64_t>(m0) * g.Kb;
    const char *baseB = g.Bm + static_cast<int64_t>(n0) * g.Kb;
    uint32_t offa[PA], offb[PB];
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int row = lr + RPP * i;
        offa[i] = static_cast<uint32_t>(m0 + row < g.M ? row : 0) * static_cast<uint32_t>(g.Kb);
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {
        const int row = lr + RPP * j;
        offb[j] = static_cast<uint32_t>(n0 + row < g.N ? row : 0) * static_cast<uint32_t>(g.Kb);
    }

    typename Mma<KIND>::acc_t acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::zero();

    u32x4 ra[PA], rb[PB];
    bool keepN = true;                 // TAIL, spread schedule: the flag of the step being loaded
    bool keepA = true, keepB = true;   // TAIL: whether this thread's chunk of the step in ra / rb lies inside the row
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    // k steps of this workgroup: all of them, or the split's share [kbeg, kbeg + nk)
    const int nk_all = (g.Kb + KCH * 16 - 1) / (KCH * 16);
    const int split = bid / (g.tiles_m * g.tiles_n);
    const int kbeg = static_cast<int>(static_cast<int64_t>(nk_all) * split / g.splits);
    const int nk = static_cast<int>(static_cast<int64_t>(nk_all) * (split + 1) / g.splits) - kbeg;

    // Step KT of k into registers (A rows, then Bm rows) with raw buffer loads: the address is
    // (tile base in the resource) + (per-thread row offset, a loop-invariant VGPR) + (k offset, an
    // SGPR), so no vector arithmetic is spent on addresses inside the loop.  With a ragged last
    // step (TAIL) chunks past the end of the row are read from the row's last chunk instead (in
    // bounds) and replaced by zeros when the registers are written to LDS.
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(baseA), 0, 0x7FFFFFFF, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(baseB), 0, 0x7FFFFFFF, 0x00020000);
#define HLQ_KOFS(KT)                                                                                          \
        const int kuni = (kbeg + (KT)) * (KCH * 16);      /* wave-uniform: lives in an SGPR */                \
        const bool kok = !TAIL || kuni + lc * 16 < g.Kb;                                                      \
        const uint32_t kfix = TAIL ? static_cast<uint32_t>(kok ? lc * 16 : g.Kb - 16 - kuni) : lc * 16u;
#define HLQ_LOAD_GLOBAL_A(KT)                                                                                 \
    {                                                                                                         \
        HLQ_KOFS(KT)                                                                                          \
        _Pragma("unroll") for (int i = 0; i < PA; ++i) {                                                      \
            ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsA, offa[i] + kfix, kuni, 0);                      \
        }                                                                                                     \
        keepA = kok;   /* applied when the registers are published, not here: no wait on the load */          \
    }
#define HLQ_LOAD_GLOBAL_B(KT)                                                                                 \
    {                                                                                                         \
        HLQ_KOFS(KT)                                                                                          \
        _Pragma("unroll") for (int j = 0; j < PB; ++j) {                                                      \
            rb[j] = __builtin_amdgcn_raw_buffer_load_b128(rsB, offb[j] + kfix, kuni, 0);                      \
        }                                                                                                     \
        keepB = kok;                                                                                          \
    }
    // LDS addressing.  Every address is (one per-lane register) + (compile-time immediate): the
    // swizzle only involves the low four row bits, so the i-th 32-row group is a constant 4 KB
    // further, and the stage is a single bit (64 KB) toggled by xor once per step.  No address
    // arithmetic is left between the MFMAs.
    static_assert(RPP == 32 && KCH == 8, "LDS address immediates below assume 32 rows x 128 B per staging pass");
    char *const ldsb = reinterpret_cast<char *>(lds);
    constexpr uint32_t STAGE_BYTES = STAGE * 16u;
    static_assert((STAGE_BYTES & (STAGE_BYTES - 1)) == 0, "stage toggling by xor needs a power-of-two stage");
    const int fr = lane & 31;   // row within a 32-row MFMA operand
    const int fh = lane >> 5;   // which 16-B half of the 32-B k slice
    uint32_t wr_off = lds_chunk<KCH>(lr, lc) * 16u + STAGE_BYTES;   // staging writes go to the other stage
    uint32_t rdA[NS], rdB[NS];                                      // fragment reads, current stage
#pragma unroll
    for (int ks = 0; ks < NS; ++ks) {
        rdA[ks] = lds_chunk<KCH>(wave_m * (32 * WM) + fr, ks * 2 + fh) * 16u;
        rdB[ks] = (BM * KCH + lds_chunk<KCH>(wave_n * (32 * WN) + fr, ks * 2 + fh)) * 16u;
    }
#define HLQ_STORE_LDS_A()                                                                                     \
    {                                                                                                         \
        _Pragma("unroll") for (int i = 0; i < PA; ++i)                                                        \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + i * (RPP * KCH * 16)) = (!TAIL || keepA) ? ra[i] : zero4; \
    }
#define HLQ_STORE_LDS_B()                                                                                     \
    {                                                                                                         \
        _Pragma("unroll") for (int j = 0; j < PB; ++j)                                                        \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + (BM * KCH * 16) + j * (RPP * KCH * 16)) =              \
                (!TAIL || keepB) ? rb[j] : zero4;                                                             \
    }
    u32x4 fa[2][WM], fb[2][WN];
#define HLQ_READ_FRAGS(BUF, KS)                                                                               \
    {   /* in the order the MFMAs consume them: fa[0] with every fb[j] first */                               \
        fb[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS]);                                        \
        fa[BUF][0] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS]);                                        \
        _Pragma("unroll") for (int j = 1; j < WN; ++j)                                                        \
            fb[BUF][j] = *reinterpret_cast<const u32x4 *>(ldsb + rdB[KS] + j * (32 * KCH * 16));              \
        _Pragma("unroll") for (int i = 1; i < WM; ++i)                                                        \
            fa[BUF][i] = *reinterpret_cast<const u32x4 *>(ldsb + rdA[KS] + i * (32 * KCH * 16));              \
    }
    // one fragment / one staging register at a time, for the schedule that spreads them out
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
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + (W_) * (RPP * KCH * 16)) = (!TAIL || keepA) ? ra[(W_) < PA ? (W_) : 0] : zero4; \
        else                                                                                                  \
            *reinterpret_cast<u32x4 *>(ldsb + wr_off + (BM * KCH * 16) + ((W_) - PA) * (RPP * KCH * 16)) =    \
                (!TAIL || keepB) ? rb[(W_) >= PA ? (W_) - PA : 0] : zero4;                                    \
    }
#define HLQ_LOAD_ONE(W_, KT)                                                                                  \
    {                                                                                                         \
        HLQ_KOFS(KT)                                                                                          \
        if ((W_) < PA) ra[(W_) < PA ? (W_) : 0] = __builtin_amdgcn_raw_buffer_load_b128(rsA, offa[(W_) < PA ? (W_) : 0] + kfix, kuni, 0); \
        else rb[(W_) >= PA ? (W_) - PA : 0] = __builtin_amdgcn_raw_buffer_load_b128(rsB, offb[(W_) >= PA ? (W_) - PA : 0] + kfix, kuni, 0); \
        keepN = kok;                                                                                          \
    }
#define HLQ_TOGGLE_STAGE()                                                                                    \
    {                                                                                                         \
        _Pragma("unroll") for (int ks = 0; ks < NS; ++ks) { rdA[ks] ^= STAGE_BYTES; rdB[ks] ^= STAGE_BYTES; } \
    }

    // The loop body is branch-free: past the end, steps are clamped to the last one, whose data is
    // loaded, published and fetched again but never multiplied.
    //
    // Step kt, sub-step ks:
    //   every ks     read the fragments of the next sub-step (the next step's first one for the
    //                last ks, from the other LDS stage) under this sub-step's MFMAs
    //   ks = 0       publish the A rows of step kt+1 (in registers since step kt-1), then load
    //                the A rows of step kt+2 into the same registers
    //   ks = 1       the same for the Bm rows
    //   ks = NS-2    barrier at its end: step kt+1 is complete in LDS, and every wavefront has
    //                finished reading the stage that step kt+2 will overwrite
    // prologue: step 0 straight into stage 0, step 1 into registers
    HLQ_LOAD_GLOBAL_A(0)
    HLQ_LOAD_GLOBAL_B(0)
    wr_off ^= STAGE_BYTES;
    HLQ_STORE_LDS_A()
    HLQ_STORE_LDS_B()
    wr_off ^= STAGE_BYTES;
    const bool one_step = nk == 1;
    if (!one_step) {
        HLQ_LOAD_GLOBAL_A(1)
        HLQ_LOAD_GLOBAL_B(1)
    }
    lds_barrier();
    u32x4 ea[2][WM][2], pb[2];    // packed codes: expanded A operands and first B operand of the coming sub-step
    if (one_step) {
        // A reduction of one step (the 4-bit codes of up to 256 out-features, a finely split k):
        // there is no pipeline to keep full.  The sub-steps that hold data are multiplied straight
        // from stage 0 (the rest of a ragged step is zeros), nothing is staged or loaded again.
        const int bytes = g.Kb - kbeg * (KCH * 16);
        const int nsub = bytes >= KCH * 16 ? NS : (bytes + 31) / 32;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            if (ks < nsub) {
                HLQ_READ_FRAGS(0, ks)
                if constexpr (KIND == 2) {
#pragma unroll
                    for (int i = 0; i < WM; ++i) Mma<2>::expand(fa[0][i], ea[0][i][0], ea[0][i][1]);
#pragma unroll
                    for (int j = 0; j < WN; ++j) {
                        Mma<2>::expand(fb[0][j], pb[0], pb[1]);
#pragma unroll
                        for (int i = 0; i < WM; ++i) acc[i][j] = Mma<2>::mma(pb[0], ea[0][i][0], acc[i][j]);
#pragma unroll
                        for (int i = 0; i < WM; ++i) acc[i][j] = Mma<2>::mma(pb[1], ea[0][i][1], acc[i][j]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::mma(fb[0][j], fa[0][i], acc[i][j]);
                }
            }
        }
    } else {
        HLQ_READ_FRAGS(0, 0)
        if constexpr (KIND == 2) {
#pragma unroll
            for (int i = 0; i < WM; ++i) Mma<2>::expand(fa[0][i], ea[0][i][0], ea[0][i][1]);
            Mma<2>::expand(fb[0][0], pb[0], pb[1]);
        }
    }
    constexpr int MPS = KIND == 2 ? 2 : 1;   // MFMAs per accumulator and sub-step
    constexpr bool SPREAD = KIND != 2 && WM == 4 && WN == 4;   // schedule with the staging writes spread out
    static_assert(!SPREAD || (PA == 8 && PB == 8), "the spread schedule publishes 8 + 8 staging registers");

    static_assert(NS == 4, "the staging schedule below is written for four sub-steps per step");

    for (int kt = 0; kt < (one_step ? 0 : nk); ++kt) {
        const int kt2 = kt + 2 < nk ? kt + 2 : nk - 1;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            const int cur = ks & 1;
            if constexpr (SPREAD) {
                // LDS writes in consecutive MFMA slots hold the MFMA stream up (measured: ~17 cycles
                // each), one write per two MFMAs costs nothing.  So the 16 staging writes of a step go
                // out one per two MFMAs over the first three sub-steps (6 + 6 + 4), between the
                // fragment reads, each followed one slot later by the global load that refills its
                // register.  Memory instructions are written here in the order they are to issue: LDS
                // accesses keep their program order.
                const int WC = ks == 0 ? 6 : (ks == 1 ? 6 : (ks == 2 ? 4 : 0));   // writes of this sub-step
                const int W0 = ks == 0 ? 0 : (ks == 1 ? 6 : 12);                   // first of them
                if (ks == NS - 1) HLQ_TOGGLE_STAGE()
#pragma unroll
                for (int q = 0; q < WM * WN; ++q) {
                    if (q < WM + WN) {
                        if (ks < NS - 1) HLQ_READ_ONE(cur ^ 1, ks + 1, q)
                        else HLQ_READ_ONE(cur ^ 1, 0, q)
                    }
                    if ((q & 1) && (q >> 1) < WC) HLQ_STORE_ONE(W0 + (q >> 1))
                    if (!(q & 1) && q >= 2 && ((q - 2) >> 1) < WC) HLQ_LOAD_ONE(W0 + ((q - 2) >> 1), kt2)
                }
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::mma(fb[cur][j], fa[cur][i], acc[i][j]);
#pragma unroll
                for (int q = 0; q < WM * WN; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (q < WM + WN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    if ((q & 1) && (q >> 1) < WC) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                    if (!(q & 1) && q >= 2 && ((q - 2) >> 1) < WC) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
                if (ks == NS - 2) {
                    wr_off ^= STAGE_BYTES;
                    keepA = keepB = keepN;
                }
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
                if (KIND != 2) HLQ_TOGGLE_STAGE()   // from here on this wavefront reads the next step's stage
                HLQ_READ_FRAGS(cur ^ 1, 0)
            }
            if constexpr (KIND == 2) {
                // packed codes: every fragment expands to two MFMA operands.  The A operands of this
                // sub-step and its first B operand were expanded under the previous sub-step's MFMAs
                // (ea[cur], pb); the other B operands are expanded here, one ahead of their use, and
                // so are the next sub-step's A operands: no MFMA waits for a burst of vector work.
                u32x4 eb[2][2];
                eb[0][0] = pb[0];
                eb[0][1] = pb[1];
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    if (j + 1 < WN) Mma<2>::expand(fb[cur][j + 1], eb[(j + 1) & 1][0], eb[(j + 1) & 1][1]);
#pragma unroll
                    for (int i = 0; i < WM; ++i) acc[i][j] = Mma<2>::mma(eb[j & 1][0], ea[cur][i][0], acc[i][j]);
#pragma unroll
                    for (int i = 0; i < WM; ++i) acc[i][j] = Mma<2>::mma(eb[j & 1][1], ea[cur][i][1], acc[i][j]);
                }
#pragma unroll
                for (int i = 0; i < WM; ++i) Mma<2>::expand(fa[cur ^ 1][i], ea[cur ^ 1][i][0], ea[cur ^ 1][i][1]);
                Mma<2>::expand(fb[cur ^ 1][0], pb[0], pb[1]);
                if (ks == NS - 1) {
                    // loop-carried: keep the compiler from moving these expansions to the top of the
                    // next iteration (it would carry the packed registers over instead), where they
                    // would stand in front of the first MFMA
#pragma unroll
                    for (int i = 0; i < WM; ++i) {
                        asm("" : "+v"(ea[cur ^ 1][i][0]));
                        asm("" : "+v"(ea[cur ^ 1][i][1]));
                    }
                    asm("" : "+v"(pb[0]));
                    asm("" : "+v"(pb[1]));
                }
            } else {
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::mma(fb[cur][j], fa[cur][i], acc[i][j]);
            }
            if (ks == 0) {
                HLQ_STORE_LDS_A()
                HLQ_LOAD_GLOBAL_A(kt2)
            }
            if (ks == 1) {
                HLQ_STORE_LDS_B()
                HLQ_LOAD_GLOBAL_B(kt2)
                wr_off ^= STAGE_BYTES;
            }
            // Issue order within the sub-step.  The fragment reads are threaded between the first
            // half of the MFMAs, so that the last of them has a quarter of a step to return before
            // anything waits on it (the next sub-step's first MFMA, the barrier, the loop's back
            // edge).  LDS writes may not pass the reads (same array): a staging sub-step threads its
            // LDS writes + global loads between the second half of the MFMAs.
            constexpr int VPS = KIND == 2 ? 12 * (WM + WN) / ((WM * WN) / 1) : 0;   // expansion instructions per slot
#pragma unroll
            for (int q = 0; q < (WM * WN) / 2; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, MPS, 0);                         // MFMA(s)
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * (WM + WN) / (WM * WN), 0);   // fragment reads
                if (VPS) __builtin_amdgcn_sched_group_barrier(0x002, VPS, 0);                // expansions
            }
#pragma unroll
            for (int q = 0; q < (WM * WN) / 2; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, MPS, 0);
                if (VPS) __builtin_amdgcn_sched_group_barrier(0x002, VPS, 0);
                if (ks < 2) {
                    __builtin_amdgcn_sched_group_barrier(0x200, 2 * PA / (WM * WN), 0);      // LDS writes
                    __builtin_amdgcn_sched_group_barrier(0x020, 2 * PA / (WM * WN), 0);      // global loads
                }
            }
            // packed codes: the address toggle is moved out of the last sub-step, which is busy enough
            if (KIND == 2 && ks == NS - 2) HLQ_TOGGLE_STAGE()
            __builtin_amdgcn_sched_barrier(0);
            if (ks == NS - 2) {              // after this sub-step's last MFMA has been issued
                lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
#undef HLQ_KOFS
#undef HLQ_LOAD_GLOBAL_A
#undef HLQ_LOAD_GLOBAL_B
#undef HLQ_STORE_LDS_A
#undef HLQ_STORE_LDS_B
#undef HLQ_READ_FRAGS
#undef HLQ_TOGGLE_STAGE
#undef HLQ_READ_ONE
#undef HLQ_STORE_ONE
#undef HLQ_LOAD_ONE

    // ---- epilogue ----
    __syncthreads();   // all fragment reads are done: LDS is free for staging C
    const int wm0 = m0 + wave_m * (32 * WM), wn0 = n0 + wave_n * (32 * WN);
    char *slab = reinterpret_cast<char *>(lds) + wave * EpiSlab<WN>::BYTES;   // wavefront-private
    // one uniform test selects straight-line code without per-store predicates for interior tiles
    const bool interior = (m0 + BM <= g.M) && (n0 + BN <= g.N) && ((g.N & 7) == 0);
    if (OUT == 2) {
        if (interior) store_raw<KIND, WM, WN, false>(acc, g.acc, g.M, g.N, wm0, wn0, lane);
        else store_raw<KIND, WM, WN, true>(acc, g.acc, g.M, g.N, wm0, wn0, lane);
    } else if (OUT == 3) {
        int32_t *part = g.partial + static_cast<int64_t>(split) * g.M * g.N;
        if (interior) store_raw<KIND, WM, WN, false>(acc, part, g.M, g.N, wm0, wn0, lane);
        else store_raw<KIND, WM, WN, true>(acc, part, g.M, g.N, wm0, wn0, lane);
    } else {
        if (interior) store_scaled<KIND, WM, WN, OUT == 1, false>(acc, g.C, g.M, g.N, g.sA, g.sB, g.alpha, wm0, wn0, lane, slab);
        else store_scaled<KIND, WM, WN, OUT == 1, true>(acc, g.C, g.M, g.N, g.sA, g.sB, g.alpha, wm0, wn0, lane, slab);
    }
}

}  // namespace hlq
