// Diagnostic: sustained MFMA issue rate of the chip at its running clock, measured with a
// register-resident loop (no LDS, no memory).  Gives the ceiling the matrix products can be priced
// against besides the datasheet peak.
#include "hlq_kernels.hpp"

namespace hlq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef int v8i __attribute__((ext_vector_type(8)));

template <int KIND>
__global__ __launch_bounds__(256) void k_mfma_probe(int iters, float *sink)
{
    const int lane = threadIdx.x;
    if (KIND == 0) {
        // a different pseudo-random operand pair for each of the eight MFMAs in flight, so that
        // consecutive MFMAs toggle the multipliers as real data does (constant operands draw less
        // power and clock higher than any product can)
        v4i a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[i][e] = static_cast<int>(0x9E3779B9u * static_cast<unsigned>(lane * 37 + i * 11 + e + 1));
                b[i][e] = static_cast<int>(0x85EBCA6Bu * static_cast<unsigned>(lane * 53 + i * 7 + e + 3));
            }
        v16i acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = v16i{0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[i], acc[i], 0, 0, 0);
        }
        int s = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
        if (s == 0x7fffffff) sink[0] = static_cast<float>(s);
    } else if (KIND == 5) {
        // bf16 on the 16x16x32 shape (half the flops per instruction, a quarter of the accumulator
        // registers): the same operand recipe as KIND 1
        typedef float v4f __attribute__((ext_vector_type(4)));
        v8bf a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned ha = 0x9E3779B9u * static_cast<unsigned>(lane * 37 + i * 11 + e + 1);
                const unsigned hb = 0x85EBCA6Bu * static_cast<unsigned>(lane * 53 + i * 7 + e + 3);
                a[i][e] = static_cast<__bf16>((static_cast<int>(ha >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
                b[i][e] = static_cast<__bf16>((static_cast<int>(hb >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
            }
        v4f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = v4f{0.0f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)   // written out: the builtin's accumulator tuples get copied around every iteration
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a[i]), "v"(b[i]));
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3];
        if (s == 12345.678f) sink[0] = s;
    } else if (KIND == 6 || KIND == 7 || KIND == 8 || KIND == 9) {
        // int8 operands as the g_x product has them: 4-bit codes in [-7, 7], KIND 7 times 16 (a nibble
        // in the high half of its byte, what the packed-code kernel feeds), KIND 8 as plain small
        // integers; KIND 6: random bytes on the 16x16x64 shape, KIND 9: the codes times 16 on that shape
        typedef int v4i32 __attribute__((ext_vector_type(4)));
        v4i a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                unsigned ha = 0x9E3779B9u * static_cast<unsigned>(lane * 37 + i * 11 + e + 1);
                unsigned hb = 0x85EBCA6Bu * static_cast<unsigned>(lane * 53 + i * 7 + e + 3);
                if (KIND != 6) {
                    constexpr bool HI = KIND == 7 || KIND == 9;
                    unsigned wa = 0, wb = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int ca = static_cast<int>((ha >> (8 * q)) & 0xFF) % 15 - 7;
                        const int cb = static_cast<int>((hb >> (8 * q)) & 0xFF) % 15 - 7;
                        wa |= (static_cast<unsigned>(HI ? ca * 16 : ca) & 0xFFu) << (8 * q);
                        wb |= (static_cast<unsigned>(HI ? cb * 16 : cb) & 0xFFu) << (8 * q);
                    }
                    ha = wa;
                    hb = wb;
                }
                a[i][e] = static_cast<int>(ha);
                b[i][e] = static_cast<int>(hb);
            }
        if (KIND == 6 || KIND == 9) {
            v4i32 acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = v4i32{0};
            for (int it = 0; it < iters; ++it) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a[i]), "v"(b[i]));
            }
            int s = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3];
            if (s == 0x7fffffff) sink[0] = static_cast<float>(s);
        } else {
            v16i acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = v16i{0};
            for (int it = 0; it < iters; ++it) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[i], acc[i], 0, 0, 0);
            }
            int s = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
            if (s == 0x7fffffff) sink[0] = static_cast<float>(s);
        }
    } else if (KIND >= 2) {
        // 32x32x64 f8f6f4 MFMA: KIND 2 = fp8 (e4m3), 3 = fp6 (e2m3), 4 = fp4 (e2m1) operands, unit scales
        constexpr int FMT = KIND == 2 ? 0 : (KIND == 3 ? 2 : 4);
        v8i a, b;
#pragma unroll
        for (int e = 0; e < 8; ++e) { a[e] = 0x12345678 * (lane + e + 1); b[e] = 0x9E3779B9 * (lane + 3 * e + 7); }
        v16f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = v16f{0.0f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], FMT, FMT, 0, 127, 0, 127);
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
        if (s == 12345.678f) sink[0] = s;
    } else {
        // as above: eight different operand pairs, values of mixed sign and magnitude in (-2, 2)
        v8bf a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned ha = 0x9E3779B9u * static_cast<unsigned>(lane * 37 + i * 11 + e + 1);
                const unsigned hb = 0x85EBCA6Bu * static_cast<unsigned>(lane * 53 + i * 7 + e + 3);
                a[i][e] = static_cast<__bf16>((static_cast<int>(ha >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
                b[i][e] = static_cast<__bf16>((static_cast<int>(hb >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
            }
        v16f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = v16f{0.0f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i], 0, 0, 0);
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
        if (s == 12345.678f) sink[0] = s;
    }
}

hipError_t launch_mfma_probe(int kind, int blocks, int iters, float *sink, hipStream_t st)
{
    switch (kind) {
        case 0: hipLaunchKernelGGL(k_mfma_probe<0>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 1: hipLaunchKernelGGL(k_mfma_probe<1>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 2: hipLaunchKernelGGL(k_mfma_probe<2>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 3: hipLaunchKernelGGL(k_mfma_probe<3>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 4: hipLaunchKernelGGL(k_mfma_probe<4>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 5: hipLaunchKernelGGL(k_mfma_probe<5>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 6: hipLaunchKernelGGL(k_mfma_probe<6>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 7: hipLaunchKernelGGL(k_mfma_probe<7>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        case 9: hipLaunchKernelGGL(k_mfma_probe<9>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
        default: hipLaunchKernelGGL(k_mfma_probe<8>, dim3(blocks), dim3(256), 0, st, iters, sink); break;
    }
    return hipGetLastError();
}

}  // namespace hlq
