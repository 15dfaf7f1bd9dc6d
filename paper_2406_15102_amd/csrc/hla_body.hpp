// Device body of K3 (see k_hla.hip): workgroup (bx, by) of 256 threads projects token blocks
// 4 by .. 4 by + 3 of the 64 * (128 / B) features starting at bx * 64 * (128 / B).
//
// Where the rows come from is a template argument: DenseRows reads a row-major [N, D] tensor;
// ConvRows reads the column matrix of a channels-last image without it ever being stored
// (arXiv 2406.15102, Sec. 3.1: the spatial positions of a convolution are the sequence) -- a lane's
// 128 / B adjacent columns are channels of one filter tap, fixed for the lane, and the B consecutive
// rows are consecutive output positions, stepped from one division per block.
#pragma once
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

template <typename Tin> struct DenseRows {
    const Tin *T;
    int64_t D;
    template <int B, int CPL> __device__ __forceinline__ void load_block(int64_t row0, int col0, float *v) const
    {
#pragma unroll
        for (int j = 0; j < B; ++j) Loader<Tin, CPL>::load(T + (row0 + j) * D + col0, v + j * CPL);
    }
};

// needs C % CPL == 0 (a lane's columns stay inside one tap) and N < 2^31
template <typename Tin> struct ConvRows {
    const Tin *X;
    ConvShape g;
    template <int B, int CPL> __device__ __forceinline__ void load_block(int64_t row0, int col0, float *v) const
    {
        const int tap = col0 / g.C, c = col0 - tap * g.C;
        const int ky = tap / g.kw, kx = tap - ky * g.kw;
        const int dy = ky * g.dh - g.ph, dx = kx * g.dw - g.pw;
        const uint32_t t = static_cast<uint32_t>(row0);
        int wo = static_cast<int>(t % static_cast<uint32_t>(g.Wo));
        const uint32_t t2 = t / static_cast<uint32_t>(g.Wo);
        int ho = static_cast<int>(t2 % static_cast<uint32_t>(g.Ho));
        int64_t n = t2 / static_cast<uint32_t>(g.Ho);
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int hi = ho * g.sh + dy, wi = wo * g.sw + dx;
            // a tap outside the image loads the nearest pixel instead (always a valid address, so the
            // B loads carry no branch and stay in flight together) and is zeroed afterwards
            const bool ok = hi >= 0 && hi < g.H && wi >= 0 && wi < g.W;
            const int hc = min(max(hi, 0), g.H - 1), wc = min(max(wi, 0), g.W - 1);
            Loader<Tin, CPL>::load(X + ((n * g.H + hc) * g.W + wc) * g.C + c, v + j * CPL);
#pragma unroll
            for (int k = 0; k < CPL; ++k) v[j * CPL + k] = ok ? v[j * CPL + k] : 0.0f;
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) {
                    ho = 0;
                    ++n;
                }
            }
        }
    }
};

// Workgroup l of a K3 job -> (column strip bx, group of 256/B token blocks by): grp consecutive by of
// one strip on one XCD (l mod 8), one after the other.  by may come out past the last group: the
// bodies return for those.
__device__ __forceinline__ void hla_job_map(int l, int gx, int grp, int &bx, int &by)
{
    const int t = l >> 3, u = (l & 7) + 8 * (t / grp);
    bx = u % gx;
    by = grp * (u / gx) + t % grp;
}

// LM: lanes side by side as a multiple of hla_lanes(B) -- 1 for the stand-alone shape (B lanes x 256/B token
// blocks), 2 for the workgroups that share their rows of G with K1 through one XCD's L2
// (2 B lanes = 256 columns x 128/B token blocks = 128 rows).
template <int B, int BASIS, typename Src, int LM = 1>
__device__ __forceinline__ void hla_body_src(const Src &src, int64_t N, int D, int r, bf16_t *__restrict__ ThatT,
                                             float *__restrict__ coeffT, int bx, int by)
{
    constexpr int CPL = 128 / B;
    constexpr int L = hla_lanes(B) * LM, NB = 256 / L;
    static_assert(NB >= 1 && L * NB == 256, "a K3 workgroup is 256 lanes");
    const int tid = threadIdx.x;
    const int col0 = (bx * L + tid % L) * CPL;
    const int64_t nblk = N / B;
    const int64_t Kc = nblk * r;
    const int64_t blk = static_cast<int64_t>(by) * NB + tid / L;
    if (col0 >= D || blk >= nblk) return;

    float v[B * CPL];
    src.template load_block<B, CPL>(blk * B, col0, v);
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

template <typename Tin, int B, int BASIS, int LM = 1>
__device__ __forceinline__ void hla_body(const Tin *__restrict__ T, int64_t N, int D, int r, bf16_t *__restrict__ ThatT,
                                         float *__restrict__ coeffT, int bx, int by)
{
    hla_body_src<B, BASIS, DenseRows<Tin>, LM>(DenseRows<Tin>{T, D}, N, D, r, ThatT, coeffT, bx, by);
}

// ---- integer g_w list: pass 1 (column maxima of the kept coefficients) and pass 2 (int8 codes) ----
template <int B, int BASIS, typename Src>
__device__ __forceinline__ void hla_absmax_body_src(const Src &src, int64_t N, int D, int r,
                                                    uint32_t *__restrict__ amax_bits, int bx, int by)
{
    constexpr int CPL = 128 / B, L = hla_lanes(B), NB = hla_blocks(B);
    __shared__ float s_max[NB][L * CPL];
    const int tid = threadIdx.x, grp = tid / L, sub = tid % L;
    const int col0 = (bx * L + sub) * CPL;
    const int64_t nblk = N / B;
    const int64_t blk = static_cast<int64_t>(by) * NB + grp;
    float cmax[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) cmax[c] = 0.0f;
    if (col0 < D && blk < nblk) {
        float v[B * CPL];
        src.template load_block<B, CPL>(blk * B, col0, v);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            fwht_regs<B, CPL>(v + c);
#pragma unroll
            for (int k = 0; k < B; ++k)
                if (k < r) cmax[c] = fmaxf(cmax[c], fabsf(v[kept_row<B, BASIS>(k) * CPL + c]));
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
        if (col < D && m > 0.0f) atomicMax(amax_bits + col, __float_as_uint(m));
    }
}

template <typename Tin, int B, int BASIS>
__device__ __forceinline__ void hla_absmax_body(const Tin *__restrict__ T, int64_t N, int D, int r,
                                                uint32_t *__restrict__ amax_bits, int bx, int by)
{
    hla_absmax_body_src<B, BASIS>(DenseRows<Tin>{T, D}, N, D, r, amax_bits, bx, by);
}

// P4: codes in [-7, 7] stored two to a byte (TqT then has Kc/2 bytes per feature; needs r % 8 == 0) -- the
// 4-bit form in which the compressed activation is kept between the passes (Sec. 6.1) -- instead of
// codes in [-127, 127], one int8 each.  Same stream, same counters, same maxima either way.
template <int B, int BASIS, bool MANT, typename Src, bool P4 = false>
__device__ __forceinline__ void hla_quantize_body_src(const Src &src, int64_t N, int D, int r,
                                                      const uint32_t *__restrict__ amax_bits, uint32_t k0, uint32_t k1,
                                                      int8_t *__restrict__ TqT, float *__restrict__ sT,
                                                      float *__restrict__ coeffT, int bx, int by)
{
    constexpr int CPL = 128 / B, L = hla_lanes(B), NB = hla_blocks(B);
    const int tid = threadIdx.x;
    const int col0 = (bx * L + tid % L) * CPL;
    const int64_t nblk = N / B;
    const int64_t Kc = nblk * r;
    const int64_t blk = static_cast<int64_t>(by) * NB + tid / L;
    if (col0 >= D || blk >= nblk) return;

    float v[B * CPL];
    src.template load_block<B, CPL>(blk * B, col0, v);
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        fwht_regs<B, CPL>(v + c);
        constexpr float QMAX = P4 ? 7.0f : 127.0f;
        const float a = __uint_as_float(amax_bits[col0 + c]);
        const float inv = absmax_to_inv(a, QMAX);
        if (blk == 0) sT[col0 + c] = absmax_to_scale(a, QMAX);
        const int64_t o = static_cast<int64_t>(col0 + c) * Kc + blk * r;          // r % 4 == 0
        const uint32_t cnt = static_cast<uint32_t>(col0 + c) * static_cast<uint32_t>(Kc >> 2) +
                             static_cast<uint32_t>((blk * r) >> 2);
        if constexpr (P4) {
#pragma unroll
            for (int k = 0; k < B; k += 8) {
                if (k < r) {
                    const uint32_t lo =
                        quant_pack4r<MANT>(v[kept_row<B, BASIS>(k + 0) * CPL + c], v[kept_row<B, BASIS>(k + 1) * CPL + c],
                                           v[kept_row<B, BASIS>(k + 2) * CPL + c], v[kept_row<B, BASIS>(k + 3) * CPL + c], inv,
                                           cnt + (k >> 2), k0, k1);
                    const uint32_t hi =
                        quant_pack4r<MANT>(v[kept_row<B, BASIS>(k + 4) * CPL + c], v[kept_row<B, BASIS>(k + 5) * CPL + c],
                                           v[kept_row<B, BASIS>(k + 6) * CPL + c], v[kept_row<B, BASIS>(k + 7) * CPL + c], inv,
                                           cnt + (k >> 2) + 1u, k0, k1);
                    *reinterpret_cast<uint32_t *>(TqT + ((o + k) >> 1)) = nibble_pack8(lo, hi);
                    if (coeffT) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) coeffT[o + k + e] = v[kept_row<B, BASIS>(k + e) * CPL + c];
                    }
                }
            }
            continue;
        }
#pragma unroll
        for (int k = 0; k < B; k += 4) {
            if (k < r) {
                *reinterpret_cast<uint32_t *>(TqT + o + k) =
                    quant_pack4r<MANT>(v[kept_row<B, BASIS>(k + 0) * CPL + c], v[kept_row<B, BASIS>(k + 1) * CPL + c],
                                       v[kept_row<B, BASIS>(k + 2) * CPL + c], v[kept_row<B, BASIS>(k + 3) * CPL + c], inv,
                                       cnt + (k >> 2), k0, k1);
                if (coeffT)
                    *reinterpret_cast<float4 *>(coeffT + o + k) =
                        make_float4(v[kept_row<B, BASIS>(k + 0) * CPL + c], v[kept_row<B, BASIS>(k + 1) * CPL + c], v[kept_row<B, BASIS>(k + 2) * CPL + c], v[kept_row<B, BASIS>(k + 3) * CPL + c]);
            }
        }
    }
}

template <typename Tin, int B, int BASIS, bool MANT = false, bool P4 = false>
__device__ __forceinline__ void hla_quantize_body(const Tin *__restrict__ T, int64_t N, int D, int r,
                                                  const uint32_t *__restrict__ amax_bits, uint32_t k0, uint32_t k1,
                                                  int8_t *__restrict__ TqT, float *__restrict__ sT,
                                                  float *__restrict__ coeffT, int bx, int by)
{
    hla_quantize_body_src<B, BASIS, MANT, DenseRows<Tin>, P4>(DenseRows<Tin>{T, D}, N, D, r, amax_bits, k0, k1, TqT, sT, coeffT,
                                                             bx, by);
}

}  // namespace hlq
