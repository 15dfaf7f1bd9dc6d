// K2 / K4 -- the two matrix products of the HLQ backward pass (arXiv 2406.15102, Sec. 6.1):
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
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 16-B chunk (first-class vector: stays in registers)
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int KIND> struct Mma;
template <> struct Mma<0> {
    typedef v16i acc_t;
    static __device__ __forceinline__ acc_t zero() { acc_t z = {0}; return z; }
    static __device__ __forceinline__ acc_t mma(const u32x4 &x, const u32x4 &y, acc_t c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(v4i, x), __builtin_bit_cast(v4i, y), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(int v) { return static_cast<float>(v); }
};
template <> struct Mma<1> {
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t zero() { acc_t z = {0.0f}; return z; }
    static __device__ __forceinline__ acc_t mma(const u32x4 &x, const u32x4 &y, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x), __builtin_bit_cast(v8bf, y), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(float v) { return v; }
};

struct GemmDev {
    const char *A;
    const char *Bm;
    int M, N;
    int Kb;            // bytes per operand row
    const float *sA;
    const float *sB;
    float alpha;
    void *C;
    int c_is_f32;
    int32_t *acc;
    int tiles_m, tiles_n;
    int splits;        // split-K: this many workgroups share a tile, each a contiguous range of k steps
    int32_t *partial;  // [splits][M][N] raw 32-bit accumulators (OUT == 3)
};

// position of 16-byte chunk c of LDS row `row` (KCH chunks per row)
template <int KCH>
__device__ __forceinline__ int lds_chunk(int row, int c)
{
    if (KCH == 8) return row * 8 + (c ^ ((row & 7) ^ ((row >> 3) & 1)));
    return row * 4 + (c ^ ((((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1)));
}

// Workgroup barrier that waits for this wavefront's LDS traffic only (global loads stay in flight).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Orders this wavefront's own LDS writes before its later LDS reads (and the reverse).
__device__ __forceinline__ void lds_wave_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// ---- epilogue helpers ------------------------------------------------------------------------
// After the MFMAs a lane holds, per accumulator (i, j) and register group vg, C[m][n .. n+3] with
// m = 32 i + (lane & 31), n = 32 j + 8 vg + 4 (lane >> 5) inside the wavefront's sub-tile.
// One wavefront per SIMD means every instruction of the epilogue is exposed, so it is kept short:
// two multiplies per value, no predicates on interior tiles.

template <int WN> struct EpiSlab {
    static constexpr int COLS = 32 * WN;
    static constexpr int PITCH_F32 = COLS * 4 + 16;   // +16 B: consecutive rows start on different banks
    static constexpr int PITCH_BF16 = COLS * 2 + 16;
    static constexpr int BYTES = 32 * PITCH_F32;      // one 32-row slab per wavefront
};

__device__ __forceinline__ int raw_bits(int v) { return v; }
__device__ __forceinline__ int raw_bits(float v) { return __builtin_bit_cast(int, v); }

// raw 32-bit accumulators (int32, or fp32 bit patterns): the parity export and the split-K
// partial results; direct 16-byte stores
template <int KIND, int WM, int WN, bool GUARD>
__device__ __forceinline__ void store_raw(typename Mma<KIND>::acc_t (&acc)[WM][WN], int32_t *out, int M, int N,
                                          int wm0, int wn0, int lane)
{
    struct { int32_t *acc; int M, N; } g = {out, M, N};
    const int fr = lane & 31, fh = lane >> 5;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int m = wm0 + i * 32 + fr;
        int32_t *row = g.acc + static_cast<int64_t>(m) * g.N + wn0 + fh * 4;
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int nl = j * 32 + vg * 8;
                if (!GUARD || (m < g.M && wn0 + nl + fh * 4 < g.N)) {
                    v4i raw = {raw_bits(acc[i][j][vg * 4 + 0]), raw_bits(acc[i][j][vg * 4 + 1]),
                               raw_bits(acc[i][j][vg * 4 + 2]), raw_bits(acc[i][j][vg * 4 + 3])};
                    *reinterpret_cast<v4i *>(row + nl) = raw;
                }
            }
    }
}

// C = alpha * sA[m] * sB[n] * acc, staged per 32-row slab through LDS so that global stores are
// 16-byte, row-contiguous pieces (a full 256-byte row segment per 16 or 8 lanes).
template <int KIND, int WM, int WN, bool F32, bool GUARD>
__device__ __forceinline__ void store_scaled(typename Mma<KIND>::acc_t (&acc)[WM][WN], void *Cout, int M, int N,
                                             const float *sA, const float *sB, float alpha, int wm0, int wn0,
                                             int lane, char *slab)
{
    struct { void *C; int M, N; const float *sA, *sB; float alpha; } g = {Cout, M, N, sA, sB, alpha};
    constexpr int COLS = EpiSlab<WN>::COLS;
    constexpr int PITCH = F32 ? EpiSlab<WN>::PITCH_F32 : EpiSlab<WN>::PITCH_BF16;
    constexpr int EPL = F32 ? 4 : 8;              // elements per 16-byte piece
    constexpr int LPR = COLS / EPL;               // lanes per row
    constexpr int RPI = 64 / LPR;                 // rows per store instruction
    const int fr = lane & 31, fh = lane >> 5;

    // column factors alpha * sB[n] for the 16 WN columns this lane owns (columns past the edge
    // read sB[0..3]: their products are never stored)
    f32x4 cs[WN][4];
    if (KIND == 1) {
        // unused
    } else if (g.sB) {
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                int n = wn0 + j * 32 + vg * 8 + fh * 4;
                if (GUARD) n = n < g.N ? n : 0;
                cs[j][vg] = *reinterpret_cast<const f32x4 *>(g.sB + n) * g.alpha;
            }
    } else {
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) cs[j][vg] = f32x4{g.alpha, g.alpha, g.alpha, g.alpha};
    }
    float sa[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        int m = wm0 + i * 32 + fr;
        if (GUARD) m = m < g.M ? m : 0;
        sa[i] = g.sA ? g.sA[m] : 1.0f;
    }

    const int rr0 = lane / LPR, cc = (lane % LPR) * EPL;
    char *wr = slab + fr * PITCH + fh * 4 * (F32 ? 4 : 2);
    const char *rd = slab + rr0 * PITCH + cc * (F32 ? 4 : 2);
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (KIND == 1) o[e] = Mma<KIND>::to_float(acc[i][j][vg * 4 + e]) * g.alpha;   // no scales on the bf16 product
                    else o[e] = Mma<KIND>::to_float(acc[i][j][vg * 4 + e]) * (sa[i] * cs[j][vg][e]);
                }
                if (F32) {
                    *reinterpret_cast<f32x4 *>(wr + (j * 32 + vg * 8) * 4) = o;
                } else {
                    u32x2 p = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
                    *reinterpret_cast<u32x2 *>(wr + (j * 32 + vg * 8) * 2) = p;
                }
            }
        lds_wave_fence();
        u32x4 v[32 / RPI];
#pragma unroll
        for (int p = 0; p < 32 / RPI; ++p) v[p] = *reinterpret_cast<const u32x4 *>(rd + p * RPI * PITCH);
        const int mbase = wm0 + i * 32 + rr0;
        char *dst = static_cast<char *>(g.C) + (static_cast<int64_t>(mbase) * g.N + wn0 + cc) * (F32 ? 4 : 2);
        const int64_t step = static_cast<int64_t>(RPI) * g.N * (F32 ? 4 : 2);
#pragma unroll
        for (int p = 0; p < 32 / RPI; ++p) {
            if (!GUARD) {
                *reinterpret_cast<u32x4 *>(dst + p * step) = v[p];
            } else {
                const int m = mbase + p * RPI, n = wn0 + cc;
                if (m < g.M) {
                    if (F32 || (g.N & 7) == 0) {
                        if (n < g.N) *reinterpret_cast<u32x4 *>(dst + p * step) = v[p];
                    } else {   // bf16 rows that are only 8-byte aligned: two halves, the last may be missing
                        const u32x2 lo = {v[p][0], v[p][1]}, hi = {v[p][2], v[p][3]};
                        if (n < g.N) *reinterpret_cast<u32x2 *>(dst + p * step) = lo;
                        if (n + 4 < g.N) *reinterpret_cast<u32x2 *>(dst + p * step + 8) = hi;
                    }
                }
            }
        }
        lds_wave_fence();
    }
}

// OUT: 0 = C in bf16, 1 = C in fp32, 2 = raw int32 accumulators (parity export),
//      3 = raw 32-bit partial accumulators of this workgroup's k range (split-K)
template <int KIND, int WM, int WN, int KCH, bool TAIL, int OUT>
__global__ __launch_bounds__(256) void k_gemm_nt(GemmDev g)
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
        const int pid = blockIdx.x % nb;           // blockIdx.x / nb is the k split
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
    bool keepA = true, keepB = true;   // TAIL: whether this thread's chunk of the step in ra / rb lies inside the row
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    // k steps of this workgroup: all of them, or the split's share [kbeg, kbeg + nk)
    const int nk_all = (g.Kb + KCH * 16 - 1) / (KCH * 16);
    const int split = blockIdx.x / (g.tiles_m * g.tiles_n);
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
    HLQ_LOAD_GLOBAL_A(nk > 1 ? 1 : 0)
    HLQ_LOAD_GLOBAL_B(nk > 1 ? 1 : 0)
    lds_barrier();
    HLQ_READ_FRAGS(0, 0)

    static_assert(NS == 4, "the staging schedule below is written for four sub-steps per step");

    for (int kt = 0; kt < nk; ++kt) {
        const int kt2 = kt + 2 < nk ? kt + 2 : nk - 1;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            const int cur = ks & 1;
            if (ks < NS - 1) {
                HLQ_READ_FRAGS(cur ^ 1, ks + 1)
            } else {
                HLQ_TOGGLE_STAGE()          // from here on this wavefront reads the next step's stage
                HLQ_READ_FRAGS(cur ^ 1, 0)
            }
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::mma(fb[cur][j], fa[cur][i], acc[i][j]);
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
#pragma unroll
            for (int q = 0; q < (WM * WN) / 2; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                           // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * (WM + WN) / (WM * WN), 0);   // fragment reads
            }
#pragma unroll
            for (int q = 0; q < (WM * WN) / 2; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (ks < 2) {
                    __builtin_amdgcn_sched_group_barrier(0x200, 2 * PA / (WM * WN), 0);      // LDS writes
                    __builtin_amdgcn_sched_group_barrier(0x020, 2 * PA / (WM * WN), 0);      // global loads
                }
            }
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

// ---- split-K: sum of the partial accumulators, then the same scaling as the direct epilogue -------
// Partials are summed in split order (integers exactly, floats in a fixed order): deterministic.
template <int KIND, bool F32>
__global__ __launch_bounds__(256) void k_splitk_reduce(const int32_t *__restrict__ partial, int splits, int M, int N,
                                                       const float *__restrict__ sA, const float *__restrict__ sB,
                                                       float alpha, void *__restrict__ C)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
    const int64_t total = static_cast<int64_t>(M) * N;
    if (e >= total) return;
    const int m = static_cast<int>(e / N), n = static_cast<int>(e % N);
    f32x4 o;
    if (KIND == 0) {
        v4i sum = {0, 0, 0, 0};
        for (int z = 0; z < splits; ++z) sum += *reinterpret_cast<const v4i *>(partial + z * total + e);
        const float sa = sA ? sA[m] : 1.0f;
        f32x4 cs = {alpha, alpha, alpha, alpha};
        if (sB) cs = *reinterpret_cast<const f32x4 *>(sB + n) * alpha;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = static_cast<float>(sum[k]) * (sa * cs[k]);
    } else {
        f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int z = 0; z < splits; ++z) sum += *reinterpret_cast<const f32x4 *>(partial + z * total + e);
        o = sum * alpha;
    }
    if (F32) {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(C) + e) = o;
    } else {
        u32x2 p = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
        *reinterpret_cast<u32x2 *>(static_cast<bf16_t *>(C) + e) = p;
    }
}

// Plan: tile size and number of k splits, from a small cost model (microseconds) fitted to
// measurements on MI355X: a 256-tile step (128 B of k) costs ~1.6 us and a tile ~12 us of fixed
// prologue/epilogue, one workgroup per compute unit; a 128-tile step ~0.5 us alone on its compute
// unit and ~0.95 us when two share it, ~6 us fixed; the split-K partials cost their HBM round trip plus a launch.
struct GemmPlan {
    bool big;
    int splits;
};

static GemmPlan plan_gemm(int M, int N, int Kb, size_t ws_bytes, bool allow_split)
{
    const int nk = (Kb + 127) / 128;
    const double mn = static_cast<double>(M) * N;
    GemmPlan best{true, 1};
    double best_t = 1e30;
    for (int big = 1; big >= 0; --big) {
        const int tile = big ? 256 : 128;
        const double tiles = static_cast<double>((M + tile - 1) / tile) * ((N + tile - 1) / tile);
        const double slots = big ? 256.0 : 512.0, fixed = big ? 12.0 : 6.0;
        for (int S = 1; S <= 16; ++S) {
            // two co-resident 128-tile workgroups share a compute unit's LDS and power: slower steps
            const double step = big ? 1.6 : (tiles * S > 256.0 ? 0.95 : 0.5);
            if (S > 1 && (!allow_split || S > nk || static_cast<double>(S) * mn * 4.0 > static_cast<double>(ws_bytes))) break;
            const double rounds = __builtin_ceil(tiles * S / slots);
            double t = rounds * (__builtin_ceil(static_cast<double>(nk) / S) * step + fixed);
            if (S > 1) t += 2.0 * S * mn * 4.0 / 5.0e6 + 4.0;
            if (t < best_t) { best_t = t; best = GemmPlan{big != 0, S}; }
        }
    }
    return best;
}

size_t gemm_ws_bytes(int kind, int M, int N, int K)
{
    const int Kb = kind == 0 ? K : 2 * K;
    const GemmPlan p = plan_gemm(M, N, Kb, ~static_cast<size_t>(0), true);
    return p.splits > 1 ? static_cast<size_t>(p.splits) * M * N * 4 : 0;
}

template <int KIND, int WM, int WN, int KCH, bool TAIL, int OUT>
static hipError_t launch_tt(const GemmArgs &a, int splits, hipStream_t st)
{
    GemmDev g;
    g.A = static_cast<const char *>(a.A);
    g.Bm = static_cast<const char *>(a.Bm);
    g.M = a.M;
    g.N = a.N;
    g.Kb = KIND == 0 ? a.K : 2 * a.K;
    g.sA = a.sA;
    g.sB = a.sB;
    g.alpha = a.alpha;
    g.C = a.C;
    g.c_is_f32 = a.c_is_f32 ? 1 : 0;
    g.acc = a.acc;
    g.tiles_m = (a.M + 64 * WM - 1) / (64 * WM);
    g.tiles_n = (a.N + 64 * WN - 1) / (64 * WN);
    g.splits = splits;
    g.partial = static_cast<int32_t *>(a.ws);
    constexpr size_t main_bytes = 2u * (64 * WM + 64 * WN) * KCH * 16u;
    constexpr size_t epi_bytes = 4u * EpiSlab<WN>::BYTES;
    constexpr size_t lds_bytes = main_bytes > epi_bytes ? main_bytes : epi_bytes;
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

template <int KIND, int WM, int WN, int KCH, int OUT>
static hipError_t launch_o(const GemmArgs &a, int splits, hipStream_t st)
{
    const int Kb = KIND == 0 ? a.K : 2 * a.K;
    return (Kb % (KCH * 16) == 0) ? launch_tt<KIND, WM, WN, KCH, false, OUT>(a, splits, st)
                                  : launch_tt<KIND, WM, WN, KCH, true, OUT>(a, splits, st);
}

template <int KIND, int WM, int WN, int KCH>
static hipError_t launch_t(const GemmArgs &a, int splits, hipStream_t st)
{
    // the raw accumulators and the scaled output are separate launches of the same product
    if (KIND == 0 && a.acc) {
        hipError_t e = launch_o<0, WM, WN, KCH, 2>(a, 1, st);
        if (e != hipSuccess || !a.C) return e;
    }
    if (splits > 1) {
        hipError_t e = launch_o<KIND, WM, WN, KCH, 3>(a, splits, st);
        if (e != hipSuccess) return e;
        const int64_t quads = (static_cast<int64_t>(a.M) * a.N + 3) / 4;
        const unsigned grid = static_cast<unsigned>((quads + 255) / 256);
        const int32_t *part = static_cast<const int32_t *>(a.ws);
        if (a.c_is_f32)
            hipLaunchKernelGGL((k_splitk_reduce<KIND, true>), dim3(grid), dim3(256), 0, st, part, splits, a.M, a.N, a.sA, a.sB, a.alpha, a.C);
        else
            hipLaunchKernelGGL((k_splitk_reduce<KIND, false>), dim3(grid), dim3(256), 0, st, part, splits, a.M, a.N, a.sA, a.sB, a.alpha, a.C);
        return hipGetLastError();
    }
    return a.c_is_f32 ? launch_o<KIND, WM, WN, KCH, 1>(a, 1, st) : launch_o<KIND, WM, WN, KCH, 0>(a, 1, st);
}

hipError_t launch_gemm_nt(int kind, const GemmArgs &a, hipStream_t st)
{
    const int Kb = kind == 0 ? a.K : 2 * a.K;
    const bool can_split = a.ws != nullptr && a.C != nullptr && (reinterpret_cast<uintptr_t>(a.ws) & 15) == 0;
    const GemmPlan p = plan_gemm(a.M, a.N, Kb, a.ws_bytes, can_split);
    if (kind == 0) return p.big ? launch_t<0, 4, 4, 8>(a, p.splits, st) : launch_t<0, 2, 2, 8>(a, p.splits, st);
    return p.big ? launch_t<1, 4, 4, 8>(a, p.splits, st) : launch_t<1, 2, 2, 8>(a, p.splits, st);
}

}  // namespace hlq
