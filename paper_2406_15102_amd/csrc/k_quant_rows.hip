// K1 -- stages 1-2 of the g_x list (arXiv 2406.15102, Sec. 6.1): block Hadamard transform of each
// row of G along d_out (Sec. 3.2, block-diagonal form), per-row absmax, 4-bit stochastic
// quantisation (Sec. 5.1), codes packed four to a dword.
//
// One row is owned by T cooperating lanes (T = 8..64 lanes of one wavefront, or the whole
// workgroup).  A lane loads chunks of 8 consecutive elements (16 B of bf16): the stride-1/2/4
// butterflies run in registers, the stride-8/16/32 ones between neighbouring lanes through
// DPP quad permutes and one ds_swizzle, so a Hadamard block of 16/32/64 spans 2/4/8 lanes.  The
// transformed row stays in registers while the absmax is reduced, then is quantised and written:
// G is read from HBM exactly once (2 B/element in, 1 B/element out).
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

constexpr int K1_MAXC = 8;  // chunks of 8 elements per lane

// PACKED: the codes are written two to a byte (4-bit codes only), O/2 bytes per row.
template <typename Tin, int B, int BLOCK, bool PACKED>
__global__ __launch_bounds__(BLOCK) void k_quant_rows(const Tin *__restrict__ G, int64_t N, int O, int T,
                                                      uint32_t k0, uint32_t k1, float qmax, int8_t *__restrict__ Gq,
                                                      float *__restrict__ sG, float *__restrict__ coeff)
{
    __shared__ float s_red[BLOCK / 64];
    const int tid = threadIdx.x;
    const int rows_per_block = BLOCK / T;
    const int g = tid % T;                       // lane index within the row's group
    const int64_t row = static_cast<int64_t>(blockIdx.x) * rows_per_block + tid / T;
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
            const uint32_t w0 = rand_word(cbase + 2u * ci, k0, k1);
            const uint32_t w1 = rand_word(cbase + 2u * ci + 1u, k0, k1);
            uint2 out;
            out.x = quant_pack4(v[m][0], v[m][1], v[m][2], v[m][3], inv, w0);
            out.y = quant_pack4(v[m][4], v[m][5], v[m][6], v[m][7], inv, w1);
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

template <typename Tin, int B, bool PACKED>
static hipError_t launch_rows_t(const void *G, int64_t N, int O, uint32_t k0, uint32_t k1, float qmax, int8_t *Gq,
                                float *sG, float *coeff, hipStream_t st)
{
    const int nch = O / 8;
    const Tin *g = static_cast<const Tin *>(G);
    if (nch <= K1_MAXC * 64) {
        int T = 8;
        while (T * K1_MAXC < nch || T < B / 8) T *= 2;   // fewest lanes that cover the row (<= 64)
        // prefer ~4 chunks per lane when the row is long enough to keep more loads in flight
        while (T < 64 && nch / T > 4) T *= 2;
        const int rows_per_block = 256 / T;
        const unsigned grid = static_cast<unsigned>((N + rows_per_block - 1) / rows_per_block);
        hipLaunchKernelGGL((k_quant_rows<Tin, B, 256, PACKED>), dim3(grid), dim3(256), 0, st, g, N, O, T, k0, k1, qmax, Gq, sG, coeff);
    } else if (nch <= K1_MAXC * 256) {
        hipLaunchKernelGGL((k_quant_rows<Tin, B, 256, PACKED>), dim3(static_cast<unsigned>(N)), dim3(256), 0, st, g, N, O, 256, k0, k1, qmax, Gq, sG, coeff);
    } else {
        hipLaunchKernelGGL((k_quant_rows<Tin, B, 1024, PACKED>), dim3(static_cast<unsigned>(N)), dim3(1024), 0, st, g, N, O, 1024, k0, k1, qmax, Gq, sG, coeff);
    }
    return hipGetLastError();
}

hipError_t launch_quant_rows(const void *G, int64_t N, int O, int B, bool is_f32, uint32_t k0, uint32_t k1,
                             float qmax, bool packed, int8_t *Gq, float *sG, float *coeff, hipStream_t st)
{
#define HLQ_ROWS_CASE(BB)                                                                                  \
    case BB:                                                                                               \
        if (packed)                                                                                        \
            return is_f32 ? launch_rows_t<float, BB, true>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st)       \
                          : launch_rows_t<bf16_t, BB, true>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st);     \
        return is_f32 ? launch_rows_t<float, BB, false>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st)          \
                      : launch_rows_t<bf16_t, BB, false>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st);
    switch (B) {
        HLQ_ROWS_CASE(16)
        HLQ_ROWS_CASE(32)
        HLQ_ROWS_CASE(64)
    }
#undef HLQ_ROWS_CASE
    return hipErrorInvalidValue;
}

}  // namespace hlq
