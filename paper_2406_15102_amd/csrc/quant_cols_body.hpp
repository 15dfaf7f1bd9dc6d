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

// `partial`: instead of merging into one maximum per column with an atomic (which needs the
// maxima zeroed by an earlier launch), the workgroup stores its own maxima as row `by` of a
// [row blocks of 4 B][I] table that pass 2 reduces; nothing needs zeroing then.
template <typename Tin, int B>
__device__ __forceinline__ void cols_absmax_body(const Tin *__restrict__ W, int O, int I, uint32_t *__restrict__ amax_bits,
                                                 int bx, int by, bool partial = false)
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
        if (col >= I) continue;
        if (partial) amax_bits[static_cast<int64_t>(by) * I + col] = __float_as_uint(m);
        else if (m > 0.0f) atomicMax(amax_bits + col, __float_as_uint(m));
    }
}

// pass 2: transform again, quantise against the column maxima, write the codes transposed.
// PACKED: the codes are written two to a byte (4-bit codes only), O/2 bytes per row of WqT.
// `parts`: rows of the table of maxima ([parts][I]; 1 = the merged maxima of the atomic pass 1).
template <typename Tin, int B, bool PACKED, bool MANT = false>
__device__ __forceinline__ void cols_quantize_body(const Tin *__restrict__ W, int O, int I,
                                                   const uint32_t *__restrict__ amax_bits, uint32_t k0, uint32_t k1,
                                                   float qmax, int8_t *__restrict__ WqT, float *__restrict__ sW,
                                                   float *__restrict__ coeffT, int bx, int by, int parts = 1)
{
    constexpr int CPL = 128 / B;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col0 = (bx * 64 + lane) * CPL;
    const int o0 = (by * 4 + wave) * B;
    if (col0 >= I || o0 >= O) return;

    float v[B * CPL];
    load_row_block<Tin, B, CPL>(W + static_cast<int64_t>(o0) * I + col0, I, v);
    // column maxima: CPL adjacent words per table row, read as vectors; non-negative floats order
    // like their bit patterns
    uint32_t abits[CPL];
    {
        typedef uint32_t uvec __attribute__((ext_vector_type(CPL)));
        uvec m = *reinterpret_cast<const uvec *>(amax_bits + col0);
        for (int p = 1; p < parts; ++p) {
            const uvec q = *reinterpret_cast<const uvec *>(amax_bits + static_cast<int64_t>(p) * I + col0);
#pragma unroll
            for (int c = 0; c < CPL; ++c) m[c] = max(m[c], q[c]);
        }
#pragma unroll
        for (int c = 0; c < CPL; ++c) abits[c] = m[c];
    }
    float inv[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const float a = __uint_as_float(abits[c]);
        inv[c] = absmax_to_inv(a, qmax);
        if (o0 == 0) sW[col0 + c] = absmax_to_scale(a, qmax);
    }
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

}  // namespace hlq
