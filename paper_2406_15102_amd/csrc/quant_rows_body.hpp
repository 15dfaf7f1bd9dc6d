// Device body of K1 (see k_quant_rows.hip), callable from any kernel whose workgroup `bx` of BLOCK
// threads is to process the rows bx * (BLOCK / T) ... of G, and the host-side choice of T.
#pragma once
#include "hlq_device.hpp"

namespace hlq {

constexpr int K1_MAXC = 8;  // chunks of 8 elements per lane

// PACKED: the codes are written two to a byte (4-bit codes only), O/2 bytes per row.
template <typename Tin, int B, int BLOCK, bool PACKED, bool MANT = false>
__device__ __forceinline__ void quant_rows_body(const Tin *__restrict__ G, int64_t N, int O, int T, uint32_t k0,
                                                uint32_t k1, float qmax, int8_t *__restrict__ Gq,
                                                float *__restrict__ sG, float *__restrict__ coeff, int bx)
{
    __shared__ float s_red[BLOCK / 64];
    const int tid = threadIdx.x;
    const int rows_per_block = BLOCK / T;
    const int g = tid % T;                       // lane index within the row's group
    const int64_t row = static_cast<int64_t>(bx) * rows_per_block + tid / T;
    const bool row_ok = row < N;
    const int nch = O >> 3;                      // 8-element chunks per row

    float v[K1_MAXC][8];
    const Tin *grow = G + (row_ok ? row : 0) * static_cast<int64_t>(O);

#pragma unroll
    for (int m = 0; m < K1_MAXC; ++m) {
        const int ci = g + m * T;
        if (ci < nch) Loader<Tin, 8>::load(grow + static_cast<int64_t>(ci) * 8, v[m]);
    }

    // Cross-lane stages leave the lane with value sign * (coefficient): see butterfly_lanes_signed.
    const float sg1 = (tid & 1) ? -1.0f : 1.0f;
    const float sg2 = (tid & 2) ? -1.0f : 1.0f;
    const float sg4 = (tid & 4) ? -1.0f : 1.0f;
    const float sign = sg1 * (B >= 32 ? sg2 : 1.0f) * (B >= 64 ? sg4 : 1.0f);

    float amax = 0.0f;
#pragma unroll
    for (int m = 0; m < K1_MAXC; ++m) {
        const int ci = g + m * T;
        // whole Hadamard blocks are either inside or outside the row: the lanes of one block
        // (aligned groups of B/8 lanes) take this branch together
        if (ci < nch) {
            fwht_regs<8, 1>(v[m]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = v[m][e];
                x = butterfly_lanes_signed<1>(x, sg1);
                if (B >= 32) x = butterfly_lanes_signed<2>(x, sg2);
                if (B >= 64) x = butterfly_lanes_signed<4>(x, sg4);
                v[m][e] = x;
                amax = fmaxf(amax, fabsf(x));
            }
        }
    }

    // absmax over the row's lanes
    if (T <= 64) {
        for (int off = 1; off < T; off *= 2) amax = fmaxf(amax, __shfl_xor(amax, off));
    } else {
        for (int off = 1; off < 64; off *= 2) amax = fmaxf(amax, __shfl_xor(amax, off));
        if ((tid & 63) == 0) s_red[tid >> 6] = amax;
        __syncthreads();
        amax = s_red[0];
#pragma unroll
        for (int w = 1; w < BLOCK / 64; ++w) amax = fmaxf(amax, s_red[w]);
    }

    if (!row_ok) return;
    const float inv = absmax_to_inv(amax, qmax) * sign;   // exact: undoes the sign the lane exchange left
    if (g == 0) sG[row] = absmax_to_scale(amax, qmax);

    const uint32_t cbase = static_cast<uint32_t>(row) * static_cast<uint32_t>(O >> 2);
    int8_t *qrow = Gq + row * static_cast<int64_t>(PACKED ? O / 2 : O);
#pragma unroll
    for (int m = 0; m < K1_MAXC; ++m) {
        const int ci = g + m * T;
        if (ci < nch) {
            uint2 out;
            out.x = quant_pack4r<MANT>(v[m][0], v[m][1], v[m][2], v[m][3], inv, cbase + 2u * ci, k0, k1);
            out.y = quant_pack4r<MANT>(v[m][4], v[m][5], v[m][6], v[m][7], inv, cbase + 2u * ci + 1u, k0, k1);
            if (PACKED) *reinterpret_cast<uint32_t *>(qrow + static_cast<int64_t>(ci) * 4) = nibble_pack8(out.x, out.y);
            else *reinterpret_cast<uint2 *>(qrow + static_cast<int64_t>(ci) * 8) = out;
            if (coeff) {
                float4 *c = reinterpret_cast<float4 *>(coeff + row * static_cast<int64_t>(O) + static_cast<int64_t>(ci) * 8);
                c[0] = make_float4(sign * v[m][0], sign * v[m][1], sign * v[m][2], sign * v[m][3]);
                c[1] = make_float4(sign * v[m][4], sign * v[m][5], sign * v[m][6], sign * v[m][7]);
            }
        }
    }
}

// Lanes per row for the 256-thread variant, or 0 if the row needs the 1024-thread one.
inline int quant_rows_lanes(int O, int B)
{
    const int nch = O / 8;
    if (nch <= K1_MAXC * 64) {
        int T = 8;
        while (T * K1_MAXC < nch || T < B / 8) T *= 2;   // fewest lanes that cover the row (<= 64)
        // prefer ~4 chunks per lane when the row is long enough to keep more loads in flight
        while (T < 64 && nch / T > 4) T *= 2;
        return T;
    }
    return nch <= K1_MAXC * 256 ? 256 : 0;
}

}  // namespace hlq
