// Device-side pieces shared by the matrix-product kernels of the HLQ backward pass: MFMA wrappers,
// the kernel argument block, LDS swizzle and barriers, and the epilogues (scaling, staging through
// LDS, row-contiguous stores).
#pragma once
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
    static __device__ __forceinline__ int raw(int v) { return v; }
};
template <> struct Mma<1> {
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t zero() { acc_t z = {0.0f}; return z; }
    static __device__ __forceinline__ acc_t mma(const u32x4 &x, const u32x4 &y, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x), __builtin_bit_cast(v8bf, y), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(float v) { return v; }
    static __device__ __forceinline__ int raw(float v) { return __builtin_bit_cast(int, v); }
};
// 4-bit codes packed two to a byte ("p4": code 2b in the low nibble of byte b, code 2b+1 in the high
// nibble, two's complement).  A nibble moved to the high half of a byte reads, as int8, as 16 x the
// code -- sign included -- so a packed dword expands to two int8 MFMA operands with three vector
// instructions and no sign extension:  x & 0xF0F0F0F0 (odd codes),  (x << 4) & 0xF0F0F0F0 (even codes).
// Both operands of a product expand the same way, so which code meets which lane of the MFMA does
// not matter.  The accumulators are 256 x the integer dot product; the factor is shifted out
// (exactly) when they are exported or scaled.
template <> struct Mma<2> {
    typedef v16i acc_t;
    static __device__ __forceinline__ acc_t zero() { acc_t z = {0}; return z; }
    static __device__ __forceinline__ acc_t mma(const u32x4 &x, const u32x4 &y, acc_t c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(v4i, x), __builtin_bit_cast(v4i, y), c, 0, 0, 0);
    }
    static __device__ __forceinline__ void expand(const u32x4 &x, u32x4 &even, u32x4 &odd)
    {
        odd = x & 0xF0F0F0F0u;
        even = (x << 4) & 0xF0F0F0F0u;
    }
    static __device__ __forceinline__ float to_float(int v) { return static_cast<float>(v >> 8); }
    static __device__ __forceinline__ int raw(int v) { return v >> 8; }
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
                    // element reads into scalars first: a bit_cast applied to a vector element
                    // expression reads element 0
                    const auto e0 = acc[i][j][vg * 4 + 0], e1 = acc[i][j][vg * 4 + 1];
                    const auto e2 = acc[i][j][vg * 4 + 2], e3 = acc[i][j][vg * 4 + 3];
                    v4i raw = {Mma<KIND>::raw(e0), Mma<KIND>::raw(e1), Mma<KIND>::raw(e2), Mma<KIND>::raw(e3)};
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

}  // namespace hlq
