// Device body of the split-K reduction: the sum of the partial accumulators of a product whose
// reduction axis was split over workgroups, then the same scaling as the direct epilogue.
// Partials are summed in split order (integers exactly, floats in a fixed order): deterministic.
// Its own kernel (k_gemm.hip) and the kernels that carry it as a side job (k_conv.hip) share it.
#pragma once
#include "gemm_common.hpp"

namespace hlq {

// KIND 0: int32 partials (the two integer products), 1: fp32 partials.  `block`: 1024 outputs each.
template <int KIND, bool F32>
__device__ __forceinline__ void splitk_reduce_body(const int32_t *__restrict__ partial, int splits, int M, int N,
                                                   const float *__restrict__ sA, const float *__restrict__ sB,
                                                   float alpha, void *__restrict__ C, int64_t block)
{
    const int64_t e = (block * 256 + threadIdx.x) * 4;
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

// the same for a kernel that learns kind and output type at run time
__device__ __forceinline__ void splitk_reduce_job(const SplitReduce &r, int64_t block)
{
    if (r.kind == 0) {
        if (r.c_is_f32) splitk_reduce_body<0, true>(r.partial, r.splits, r.M, r.N, r.sA, r.sB, r.alpha, r.C, block);
        else splitk_reduce_body<0, false>(r.partial, r.splits, r.M, r.N, r.sA, r.sB, r.alpha, r.C, block);
    } else {
        if (r.c_is_f32) splitk_reduce_body<1, true>(r.partial, r.splits, r.M, r.N, r.sA, r.sB, r.alpha, r.C, block);
        else splitk_reduce_body<1, false>(r.partial, r.splits, r.M, r.N, r.sA, r.sB, r.alpha, r.C, block);
    }
}

}  // namespace hlq
