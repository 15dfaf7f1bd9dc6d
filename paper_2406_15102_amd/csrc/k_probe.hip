// Diagnostic: sustained MFMA issue rate of the chip at its running clock, measured with a
// register-resident loop (no LDS, no memory).  Gives the ceiling the matrix products can be priced
// against besides the datasheet peak.
#include "hlq_kernels.hpp"

namespace hlq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int KIND>
__global__ __launch_bounds__(256) void k_mfma_probe(int iters, float *sink)
{
    const int lane = threadIdx.x;
    if (KIND == 0) {
        v4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {lane * 3, lane * 5, lane * 7, lane * 11};
        v16i acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = v16i{0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
        }
        int s = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
        if (s == 0x7fffffff) sink[0] = static_cast<float>(s);
    } else {
        v8bf a, b;
#pragma unroll
        for (int e = 0; e < 8; ++e) { a[e] = static_cast<__bf16>(1.0f + lane * 0.001f); b[e] = static_cast<__bf16>(0.5f); }
        v16f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = v16f{0.0f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
        if (s == 12345.678f) sink[0] = s;
    }
}

hipError_t launch_mfma_probe(int kind, int blocks, int iters, float *sink, hipStream_t st)
{
    if (kind == 0) hipLaunchKernelGGL(k_mfma_probe<0>, dim3(blocks), dim3(256), 0, st, iters, sink);
    else hipLaunchKernelGGL(k_mfma_probe<1>, dim3(blocks), dim3(256), 0, st, iters, sink);
    return hipGetLastError();
}

}  // namespace hlq
