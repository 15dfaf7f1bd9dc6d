// K1T -- stages 3-4 of the g_x list (arXiv 2406.15102, Sec. 6.1): H_O^T . W, i.e. the block
// Hadamard transform (Sec. 3.2) over groups of B consecutive ROWS of W [d_out, d_in], then 4-bit
// stochastic quantisation (Sec. 5.1) with one absmax scale per in-feature (= per column of W,
// = per row of the transposed, reduction-contiguous output WqT [d_in, d_out]).
//
// A lane owns CPL = 128/B adjacent columns and walks down the rows: B row loads of CPL elements
// give it whole Hadamard blocks in registers, so the transform needs no lane exchange.  The
// column absmax spans all of d_out, hence two passes over W:
//   pass 1  transform, per-column max over a 256-row tile      -> partial [tiles, d_in]
//   fin     max over tiles -> scale and reciprocal scale        -> sW, inv [d_in]
//   pass 2  transform again, quantise, write 64 codes per column and wave (contiguous in d_out)
// max() is order-independent, so the result does not depend on the tiling.
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

constexpr int KT_ROWS_PER_WAVE = 64;
constexpr int KT_TILE_ROWS = 4 * KT_ROWS_PER_WAVE;

template <typename Tin, int B, int CPL>
__device__ __forceinline__ void load_row_block(const Tin *base, int64_t pitch, float *v)
{
#pragma unroll
    for (int j = 0; j < B; ++j) Loader<Tin, CPL>::load(base + j * pitch, v + j * CPL);
}

template <typename Tin, int B>
__global__ __launch_bounds__(256) void k_cols_absmax(const Tin *__restrict__ W, int O, int I,
                                                     float *__restrict__ partial)
{
    constexpr int CPL = 128 / B;
    constexpr int NBW = KT_ROWS_PER_WAVE / B;
    __shared__ float s_max[4][64 * CPL];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col0 = (blockIdx.x * 64 + lane) * CPL;
    float cmax[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) cmax[c] = 0.0f;

    if (col0 < I) {
#pragma unroll 1
        for (int t = 0; t < NBW; ++t) {
            const int o0 = blockIdx.y * KT_TILE_ROWS + wave * KT_ROWS_PER_WAVE + t * B;
            if (o0 >= O) break;
            float v[B * CPL];
            load_row_block<Tin, B, CPL>(W + static_cast<int64_t>(o0) * I + col0, I, v);
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                fwht_regs<B, CPL>(v + c);
#pragma unroll
                for (int j = 0; j < B; ++j) cmax[c] = fmaxf(cmax[c], fabsf(v[j * CPL + c]));
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CPL; ++c) s_max[wave][lane * CPL + c] = cmax[c];
    __syncthreads();
    for (int idx = tid; idx < 64 * CPL; idx += 256) {
        const float m = fmaxf(fmaxf(s_max[0][idx], s_max[1][idx]), fmaxf(s_max[2][idx], s_max[3][idx]));
        const int col = blockIdx.x * 64 * CPL + idx;
        if (col < I) partial[static_cast<int64_t>(blockIdx.y) * I + col] = m;
    }
}

__global__ __launch_bounds__(256) void k_cols_finalize(const float *__restrict__ partial, int ntile, int I,
                                                       float *__restrict__ sW, float *__restrict__ inv)
{
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= I) return;
    float a = 0.0f;
    for (int t = 0; t < ntile; ++t) a = fmaxf(a, partial[static_cast<int64_t>(t) * I + col]);
    sW[col] = absmax_to_scale(a);
    inv[col] = absmax_to_inv(a);
}

template <typename Tin, int B>
__global__ __launch_bounds__(256) void k_cols_quantize(const Tin *__restrict__ W, int O, int I,
                                                       const float *__restrict__ invW, uint32_t k0, uint32_t k1,
                                                       int8_t *__restrict__ WqT, float *__restrict__ coeffT)
{
    constexpr int CPL = 128 / B;
    constexpr int NBW = KT_ROWS_PER_WAVE / B;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col0 = (blockIdx.x * 64 + lane) * CPL;
    if (col0 >= I) return;
    float inv[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) inv[c] = invW[col0 + c];

#pragma unroll 1
    for (int t = 0; t < NBW; ++t) {
        const int o0 = blockIdx.y * KT_TILE_ROWS + wave * KT_ROWS_PER_WAVE + t * B;
        if (o0 >= O) break;
        float v[B * CPL];
        load_row_block<Tin, B, CPL>(W + static_cast<int64_t>(o0) * I + col0, I, v);
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
                    const uint32_t w = rand_word(cnt + d4 * 4 + d, k0, k1);
                    out[d] = quant_pack4(v[(j + 0) * CPL + c], v[(j + 1) * CPL + c], v[(j + 2) * CPL + c],
                                         v[(j + 3) * CPL + c], inv[c], w);
                }
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
}

static inline int kt_tiles(int64_t O) { return static_cast<int>((O + KT_TILE_ROWS - 1) / KT_TILE_ROWS); }

size_t quant_cols_ws_bytes(int64_t O, int64_t I)
{
    // partial [tiles, I] fp32, then inv [I] fp32, each rounded up to 256 B
    size_t part = (static_cast<size_t>(kt_tiles(O)) * I * 4 + 255) & ~static_cast<size_t>(255);
    size_t inv = (static_cast<size_t>(I) * 4 + 255) & ~static_cast<size_t>(255);
    return part + inv;
}

template <typename Tin, int B>
static hipError_t launch_cols_t(const void *W, int O, int I, uint32_t k0, uint32_t k1, int8_t *WqT, float *sW,
                                float *coeffT, void *ws, hipStream_t st)
{
    constexpr int CPL = 128 / B;
    const int ntile = kt_tiles(O);
    float *partial = static_cast<float *>(ws);
    size_t part = (static_cast<size_t>(ntile) * I * 4 + 255) & ~static_cast<size_t>(255);
    float *inv = reinterpret_cast<float *>(static_cast<char *>(ws) + part);
    const Tin *w = static_cast<const Tin *>(W);
    dim3 grid((I + 64 * CPL - 1) / (64 * CPL), ntile);
    hipLaunchKernelGGL((k_cols_absmax<Tin, B>), grid, dim3(256), 0, st, w, O, I, partial);
    hipLaunchKernelGGL(k_cols_finalize, dim3((I + 255) / 256), dim3(256), 0, st, partial, ntile, I, sW, inv);
    hipLaunchKernelGGL((k_cols_quantize<Tin, B>), grid, dim3(256), 0, st, w, O, I, inv, k0, k1, WqT, coeffT);
    return hipGetLastError();
}

hipError_t launch_quant_cols(const void *W, int O, int I, int B, bool is_f32, uint32_t k0, uint32_t k1,
                             int8_t *WqT, float *sW, float *coeffT, void *ws, hipStream_t st)
{
#define HLQ_COLS_CASE(BB)                                                                            \
    case BB:                                                                                         \
        return is_f32 ? launch_cols_t<float, BB>(W, O, I, k0, k1, WqT, sW, coeffT, ws, st)           \
                      : launch_cols_t<bf16_t, BB>(W, O, I, k0, k1, WqT, sW, coeffT, ws, st);
    switch (B) {
        HLQ_COLS_CASE(16)
        HLQ_COLS_CASE(32)
        HLQ_COLS_CASE(64)
    }
#undef HLQ_COLS_CASE
    return hipErrorInvalidValue;
}

}  // namespace hlq
