// Device pieces of K1T (see k_quant_cols.hip) that other kernels reuse: the row-block loader and
// pass 1, the column maxima of the transformed weight.
#pragma once
#include "hlq_device.hpp"

namespace hlq {

template <typename Tin, int B, int CPL>
__device__ __forceinline__ void load_row_block(const Tin *base, int64_t pitch, float *v)
{
#pragma unroll
    for (int j = 0; j < B; ++j) Loader<Tin, CPL>::load(base + j * pitch, v + j * CPL);
}

template <typename Tin, int B>
__device__ __forceinline__ void cols_absmax_body(const Tin *__restrict__ W, int O, int I, uint32_t *__restrict__ amax_bits,
                                                 int bx, int by)
{
    constexpr int CPL = 128 / B;
    __shared__ float s_max[4][64 * CPL];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col0 = (bx * 64 + lane) * CPL;
    const int o0 = (by * 4 + wave) * B;
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
    for (int c = 0; c < CPL; ++c) s_max[wave][lane * CPL + c] = cmax[c];
    __syncthreads();
    for (int idx = tid; idx < 64 * CPL; idx += 256) {
        const float m = fmaxf(fmaxf(s_max[0][idx], s_max[1][idx]), fmaxf(s_max[2][idx], s_max[3][idx]));
        const int col = bx * 64 * CPL + idx;
        if (col < I && m > 0.0f) atomicMax(amax_bits + col, __float_as_uint(m));
    }
}

}  // namespace hlq
