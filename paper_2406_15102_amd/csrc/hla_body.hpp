// Device body of K3 (see k_hla.hip): workgroup (bx, by) of 256 threads projects token blocks
// 4 by .. 4 by + 3 of the 64 * (128 / B) features starting at bx * 64 * (128 / B).
#pragma once
#include "hlq_device.hpp"

namespace hlq {

template <typename Tin, int B, int BASIS>
__device__ __forceinline__ void hla_body(const Tin *__restrict__ T, int64_t N, int D, int r, bf16_t *__restrict__ ThatT,
                                         float *__restrict__ coeffT, int bx, int by)
{
    constexpr int CPL = 128 / B;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col0 = (bx * 64 + lane) * CPL;
    const int64_t nblk = N / B;
    const int64_t Kc = nblk * r;
    const int64_t blk = static_cast<int64_t>(by) * 4 + wave;
    if (col0 >= D || blk >= nblk) return;

    float v[B * CPL];
#pragma unroll
    for (int j = 0; j < B; ++j)
        Loader<Tin, CPL>::load(T + (blk * B + j) * static_cast<int64_t>(D) + col0, v + j * CPL);
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        fwht_regs<B, CPL>(v + c);
        const int64_t o = static_cast<int64_t>(col0 + c) * Kc + blk * r;
        if (r >= 8) {
#pragma unroll
            for (int k = 0; k < B; k += 8) {
                if (k < r) {
                    uint4 p;
                    p.x = pack_bf16(v[kept_row<B, BASIS>(k + 0) * CPL + c], v[kept_row<B, BASIS>(k + 1) * CPL + c]);
                    p.y = pack_bf16(v[kept_row<B, BASIS>(k + 2) * CPL + c], v[kept_row<B, BASIS>(k + 3) * CPL + c]);
                    p.z = pack_bf16(v[kept_row<B, BASIS>(k + 4) * CPL + c], v[kept_row<B, BASIS>(k + 5) * CPL + c]);
                    p.w = pack_bf16(v[kept_row<B, BASIS>(k + 6) * CPL + c], v[kept_row<B, BASIS>(k + 7) * CPL + c]);
                    *reinterpret_cast<uint4 *>(ThatT + o + k) = p;
                }
            }
        } else if (r == 4) {
            uint2 p;
            p.x = pack_bf16(v[kept_row<B, BASIS>(0) * CPL + c], v[kept_row<B, BASIS>(1) * CPL + c]);
            p.y = pack_bf16(v[kept_row<B, BASIS>(2) * CPL + c], v[kept_row<B, BASIS>(3) * CPL + c]);
            *reinterpret_cast<uint2 *>(ThatT + o) = p;
        } else if (r == 2) {
            *reinterpret_cast<uint32_t *>(ThatT + o) = pack_bf16(v[kept_row<B, BASIS>(0) * CPL + c], v[kept_row<B, BASIS>(1) * CPL + c]);
        } else {
            ThatT[o] = static_cast<bf16_t>(pack_bf16(v[c], 0.0f) & 0xFFFFu);
        }
        if (coeffT) {
#pragma unroll
            for (int k = 0; k < B; ++k)
                if (k < r) coeffT[o + k] = v[kept_row<B, BASIS>(k) * CPL + c];
        }
    }
}

}  // namespace hlq
