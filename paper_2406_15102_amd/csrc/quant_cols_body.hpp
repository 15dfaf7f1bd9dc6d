// Device pieces of K1T (see k_quant_cols.hip) that other kernels reuse: the row-block loader and
// pass 1, the column maxima of the transformed weight.
#pragma once
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

template <typename Tin, int B, int CPL>
__device__ __forceinline__ void load_row_block(const Tin *base, int64_t pitch, float *v)
{
#pragma unroll
    for (int j = 0; j < B; ++j) Loader<Tin, CPL>::load(base + j * pitch, v + j * CPL);
}

// pass 1: a row block per group of B lanes (256 / B groups); the groups' maxima meet in LDS and are merged
// into one maximum per column with an atomic on the bit patterns (non-negative floats order like
// their bit patterns), so the maxima must have been zeroed by an earlier launch.
template <typename Tin, int B>
__device__ __forceinline__ void cols_absmax_body(const Tin *__restrict__ W, int O, int I, uint32_t *__restrict__ amax_bits,
                                                 int bx, int by)
{
    constexpr int CPL = 128 / B, L = B, NB = 256 / B;     // lanes side by side, row blocks
    __shared__ float s_max[NB][L * CPL];
    const int tid = threadIdx.x, grp = tid / L, sub = tid % L;
    const int col0 = (bx * L + sub) * CPL;
    const int o0 = (by * NB + grp) * B;
    float cmax[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) cmax[c] = 0.0f;

    if (col0 < I && o0 < O) {
        float v[B * CPL];
        load_row_block<Tin, B, CPL>(W + static_cast<int64_t>(o0) * I + col0, I, v);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            fwht_regs<B, CPL>(v + c);
#pragma unroll
            for (int j = 0; j < B; ++j) cmax[c] = fmaxf(cmax[c], fabsf(v[j * CPL + c]));
        }
    }
#pragma unroll
    for (int c = 0; c < CPL; ++c) s_max[grp][sub * CPL + c] = cmax[c];
    __syncthreads();
    for (int idx = tid; idx < L * CPL; idx += 256) {
        float m = s_max[0][idx];
#pragma unroll
        for (int g = 1; g < NB; ++g) m = fmaxf(m, s_max[g][idx]);
        const int col = bx * L * CPL + idx;
        if (col < I && m > 0.0f) atomicMax(amax_bits + col, __float_as_uint(m));
    }
}

// One row block (B rows from o0) of CPL columns (a lane's share) from col0: transform again, quantise against the
// reciprocal scales `inv` of those columns, write the codes transposed.
// PACKED: the codes are written two to a byte (4-bit codes only), O/2 bytes per row of WqT.
template <typename Tin, int B, bool PACKED, bool MANT, int CPL = 128 / B>
__device__ __forceinline__ void cols_quantize_block(const Tin *__restrict__ W, int O, int I, const float *inv, uint32_t k0,
                                                    uint32_t k1, int8_t *__restrict__ WqT, float *__restrict__ coeffT,
                                                    int col0, int o0)
{
    float v[B * CPL];
    load_row_block<Tin, B, CPL>(W + static_cast<int64_t>(o0) * I + col0, I, v);
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        fwht_regs<B, CPL>(v + c);
        const int64_t orow = static_cast<int64_t>(col0 + c) * O + o0;
        const uint32_t cnt = static_cast<uint32_t>(col0 + c) * static_cast<uint32_t>(O >> 2) +
                             static_cast<uint32_t>(o0 >> 2);
#pragma unroll
        for (int d4 = 0; d4 < B / 16; ++d4) {
            uint32_t out[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int j = (d4 * 4 + d) * 4;
                out[d] = quant_pack4r<MANT>(v[(j + 0) * CPL + c], v[(j + 1) * CPL + c], v[(j + 2) * CPL + c],
                                            v[(j + 3) * CPL + c], inv[c], cnt + d4 * 4 + d, k0, k1);
            }
            if (PACKED)
                *reinterpret_cast<uint2 *>(WqT + orow / 2 + d4 * 8) =
                    make_uint2(nibble_pack8(out[0], out[1]), nibble_pack8(out[2], out[3]));
            else
                *reinterpret_cast<uint4 *>(WqT + orow + d4 * 16) = make_uint4(out[0], out[1], out[2], out[3]);
        }
        if (coeffT) {
#pragma unroll
            for (int j = 0; j < B; j += 4)
                *reinterpret_cast<float4 *>(coeffT + orow + j) =
                    make_float4(v[j * CPL + c], v[(j + 1) * CPL + c], v[(j + 2) * CPL + c], v[(j + 3) * CPL + c]);
        }
    }
}

// pass 2: a row block per group of B lanes against the column maxima that pass 1 merged.
template <typename Tin, int B, bool PACKED, bool MANT = false>
__device__ __forceinline__ void cols_quantize_body(const Tin *__restrict__ W, int O, int I,
                                                   const uint32_t *__restrict__ amax_bits, uint32_t k0, uint32_t k1,
                                                   float qmax, int8_t *__restrict__ WqT, float *__restrict__ sW,
                                                   float *__restrict__ coeffT, int bx, int by)
{
    constexpr int CPL = 128 / B;
    constexpr int L = B, NB = 256 / B;
    const int tid = threadIdx.x;
    const int col0 = (bx * L + tid % L) * CPL;
    const int o0 = (by * NB + tid / L) * B;
    if (col0 >= I || o0 >= O) return;
    float inv[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const float a = __uint_as_float(amax_bits[col0 + c]);
        inv[c] = absmax_to_inv(a, qmax);
        if (o0 == 0) sW[col0 + c] = absmax_to_scale(a, qmax);
    }
    cols_quantize_block<Tin, B, PACKED, MANT>(W, O, I, inv, k0, k1, WqT, coeffT, col0, o0);
}

// Both passes by one workgroup, for a small weight: the workgroup owns a strip of LG * CW columns
// over all of O (LG = 1 << lg lanes side by side: 16, 8 or 4; CW columns a lane, fewer than the
// 128/B of the two-pass kernels so that a lane's chain of loads, transform and quantisation is
// short: this job's latency is what the launch around it can end on), its 256 / LG groups of lanes
// take a row block each per round, the maxima meet in LDS, and the second pass finds the rows in
// the cache.  No other workgroup is waited for, so this can ride in a launch with anything.
template <int B> struct ColsFull {
    static constexpr int CW = B == 16 ? 4 : 2;      // columns a lane: 64 (B = 16, 32) or 128 values
};

template <typename Tin, int B, bool PACKED>
__device__ __forceinline__ void cols_full_body(const Tin *__restrict__ W, int O, int I, uint32_t k0, uint32_t k1, float qmax,
                                               int8_t *__restrict__ WqT, float *__restrict__ sW, int bx, int lg)
{
    constexpr int CW = ColsFull<B>::CW;
    __shared__ float s_strip[256 * CW];       // [group][lane of the group][column of the lane]
    const int tid = threadIdx.x, grp = tid >> lg, sub = tid & ((1 << lg) - 1), groups = 256 >> lg;
    const int col0 = ((bx << lg) + sub) * CW;
    const int nrb = O / B;
    float cmax[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) cmax[c] = 0.0f;
    if (col0 < I) {
#pragma nounroll
        for (int rb = grp; rb < nrb; rb += groups) {
            float v[B * CW];
            load_row_block<Tin, B, CW>(W + static_cast<int64_t>(rb) * B * I + col0, I, v);
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                fwht_regs<B, CW>(v + c);
#pragma unroll
                for (int j = 0; j < B; ++j) cmax[c] = fmaxf(cmax[c], fabsf(v[j * CW + c]));
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CW; ++c) s_strip[tid * CW + c] = cmax[c];
    __syncthreads();
    if (col0 >= I) return;
    // a few groups at a time: all of them in flight would cost CW registers each
#pragma unroll 4
    for (int g = 0; g < groups; ++g) {
#pragma unroll
        for (int c = 0; c < CW; ++c) cmax[c] = fmaxf(cmax[c], s_strip[((g << lg) + sub) * CW + c]);
    }
    float inv[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        inv[c] = absmax_to_inv(cmax[c], qmax);
        if (grp == 0) sW[col0 + c] = absmax_to_scale(cmax[c], qmax);
    }
#pragma nounroll
    for (int rb = grp; rb < nrb; rb += groups)
        cols_quantize_block<Tin, B, PACKED, false, CW>(W, O, I, inv, k0, k1, WqT, nullptr, col0, rb * B);
}

}  // namespace hlq
