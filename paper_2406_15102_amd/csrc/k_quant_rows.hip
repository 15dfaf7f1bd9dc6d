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
#include "quant_rows_body.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

template <typename Tin, int B, int BLOCK, bool PACKED, bool MANT>
__global__ __launch_bounds__(BLOCK) void k_quant_rows(const Tin *__restrict__ G, int64_t N, int O, int T,
                                                      uint32_t k0, uint32_t k1, float qmax, int8_t *__restrict__ Gq,
                                                      float *__restrict__ sG, float *__restrict__ coeff)
{
    quant_rows_body<Tin, B, BLOCK, PACKED, MANT>(G, N, O, T, k0, k1, qmax, Gq, sG, coeff, blockIdx.x);
}

template <typename Tin, int B, bool PACKED, bool MANT>
static hipError_t launch_rows_t(const void *G, int64_t N, int O, uint32_t k0, uint32_t k1, float qmax, int8_t *Gq,
                                float *sG, float *coeff, hipStream_t st)
{
    const Tin *g = static_cast<const Tin *>(G);
    const int T = quant_rows_lanes(O, B);
    if (T > 0 && T <= 64) {
        const int rows_per_block = 256 / T;
        const unsigned grid = static_cast<unsigned>((N + rows_per_block - 1) / rows_per_block);
        hipLaunchKernelGGL((k_quant_rows<Tin, B, 256, PACKED, MANT>), dim3(grid), dim3(256), 0, st, g, N, O, T, k0, k1, qmax, Gq, sG, coeff);
    } else if (T == 256) {
        hipLaunchKernelGGL((k_quant_rows<Tin, B, 256, PACKED, MANT>), dim3(static_cast<unsigned>(N)), dim3(256), 0, st, g, N, O, 256, k0, k1, qmax, Gq, sG, coeff);
    } else {
        hipLaunchKernelGGL((k_quant_rows<Tin, B, 1024, PACKED, MANT>), dim3(static_cast<unsigned>(N)), dim3(1024), 0, st, g, N, O, 1024, k0, k1, qmax, Gq, sG, coeff);
    }
    return hipGetLastError();
}

template <typename Tin, int B>
static hipError_t launch_rows_v(const void *G, int64_t N, int O, uint32_t k0, uint32_t k1, float qmax, bool packed,
                                bool mant, int8_t *Gq, float *sG, float *coeff, hipStream_t st)
{
    if (packed) return mant ? launch_rows_t<Tin, B, true, true>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st)
                            : launch_rows_t<Tin, B, true, false>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st);
    return mant ? launch_rows_t<Tin, B, false, true>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st)
                : launch_rows_t<Tin, B, false, false>(G, N, O, k0, k1, qmax, Gq, sG, coeff, st);
}

hipError_t launch_quant_rows(const void *G, int64_t N, int O, int B, bool is_f32, uint32_t k0, uint32_t k1,
                             float qmax, bool packed, bool mant, int8_t *Gq, float *sG, float *coeff, hipStream_t st)
{
#define HLQ_ROWS_CASE(BB)                                                                                     \
    case BB:                                                                                                  \
        return is_f32 ? launch_rows_v<float, BB>(G, N, O, k0, k1, qmax, packed, mant, Gq, sG, coeff, st)      \
                      : launch_rows_v<bf16_t, BB>(G, N, O, k0, k1, qmax, packed, mant, Gq, sG, coeff, st);
    switch (B) {
        HLQ_ROWS_CASE(16)
        HLQ_ROWS_CASE(32)
        HLQ_ROWS_CASE(64)
    }
#undef HLQ_ROWS_CASE
    return hipErrorInvalidValue;
}

}  // namespace hlq
