// K3 -- Hadamard low-rank approximation along the token axis (arXiv 2406.15102, Sec. 4 and 5.1;
// stages 1 and 3 of the g_w list of Sec. 6.1, stage 1 being what ACBP stores at forward time).
// For a tensor T [N, D] (G or X), token block b and feature j:
//     ThatT[j, b*r + k] = bf16( sum_n H[k][n] * T[b*B + n, j] ),   k < r
// with H the +-1 natural-order Walsh-Hadamard matrix of order B (Sec. 3.2): the first r of every
// B coefficients, written with the compressed token axis contiguous so that the dW product reads
// both operands reduction-major.
//
// A lane owns CPL = 128/B adjacent features and B consecutive tokens: B fully coalesced row loads
// put whole Hadamard blocks in its registers and the butterflies need no lane exchange.  A
// wavefront is one (B tokens) x (64*CPL features) unit of work, a workgroup four consecutive
// token blocks (their outputs are adjacent: 4*r contiguous values per feature).
// T is read once (2 B/element), r/B of it is written back as bf16.
#include "hla_body.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

template <typename Tin, int B, int BASIS>
__global__ __launch_bounds__(256) void k_hla(const Tin *__restrict__ T, int64_t N, int D, int r,
                                             bf16_t *__restrict__ ThatT, float *__restrict__ coeffT, int gx, int grp)
{
    int bx, by;
    hla_job_map(static_cast<int>(blockIdx.x), gx, grp, bx, by);
    hla_body<Tin, B, BASIS>(T, N, D, r, ThatT, coeffT, bx, by);
}

template <typename Tin, int B>
static hipError_t launch_hla_t(const void *T, int64_t N, int D, int r, int basis, bf16_t *ThatT, float *coeffT, hipStream_t st)
{
    constexpr int CPL = 128 / B;
    const int64_t nblk = N / B;
    const int gx = hla_grid_x(D, B), gy = hla_grid_y(N, B);
    const int grp = hla_job_grp(B, r);
    const dim3 grid(hla_job_blocks(gx, gy, grp));
    if (basis)
        hipLaunchKernelGGL((k_hla<Tin, B, 1>), grid, dim3(256), 0, st, static_cast<const Tin *>(T), N, D, r, ThatT, coeffT, gx, grp);
    else
        hipLaunchKernelGGL((k_hla<Tin, B, 0>), grid, dim3(256), 0, st, static_cast<const Tin *>(T), N, D, r, ThatT, coeffT, gx, grp);
    return hipGetLastError();
}

hipError_t launch_hla(const void *T, int64_t N, int D, int B, int r, int basis, bool is_f32, uint16_t *ThatT,
                      float *coeffT, hipStream_t st)
{
#define HLQ_HLA_CASE(BB)                                                                  \
    case BB:                                                                              \
        return is_f32 ? launch_hla_t<float, BB>(T, N, D, r, basis, ThatT, coeffT, st)            \
                      : launch_hla_t<bf16_t, BB>(T, N, D, r, basis, ThatT, coeffT, st);
    switch (B) {
        HLQ_HLA_CASE(16)
        HLQ_HLA_CASE(32)
        HLQ_HLA_CASE(64)
    }
#undef HLQ_HLA_CASE
    return hipErrorInvalidValue;
}

// ---- integer g_w path: projection + int8 quantisation (stages 1-2 and 3-4 of the g_w list) ----
// One scale per feature (= per row of the reduction-contiguous output TqT [D, N/B*r]), so the
// absmax spans the whole token axis: two passes over T, as for the weight operand of the g_x path.
//   zero    amax[D] = 0
//   pass 1  transform, max |coefficient| over the kept r per column, LDS across the workgroup's
//           four token blocks, one atomic max (on the bit pattern of a non-negative float) per column
//   pass 2  transform again, quantise the kept coefficients with qmax = 127, write r codes per
//           column and token block
__global__ __launch_bounds__(256) void k_hla_fill_u32(uint32_t *p, int n, uint32_t value)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = value;
}

template <typename Tin, int B, int BASIS>
__global__ __launch_bounds__(256) void k_hla_absmax(const Tin *__restrict__ T, int64_t N, int D, int r,
                                                    uint32_t *__restrict__ amax_bits)
{
    hla_absmax_body<Tin, B, BASIS>(T, N, D, r, amax_bits, blockIdx.x, blockIdx.y);
}

template <typename Tin, int B, int BASIS, bool MANT, bool P4 = false>
__global__ __launch_bounds__(256) void k_hla_quantize(const Tin *__restrict__ T, int64_t N, int D, int r,
                                                      const uint32_t *__restrict__ amax_bits, uint32_t k0,
                                                      uint32_t k1, int8_t *__restrict__ TqT, float *__restrict__ sT,
                                                      float *__restrict__ coeffT)
{
    // backwards (reverse_same_xcd): what the pass that took the maxima read last is what the last-level cache still holds
    const int lin = reverse_same_xcd(blockIdx.x + blockIdx.y * gridDim.x, gridDim.x * gridDim.y,
                                     N * D * static_cast<int64_t>(sizeof(Tin)));
    hla_quantize_body<Tin, B, BASIS, MANT, P4>(T, N, D, r, amax_bits, k0, k1, TqT, sT, coeffT, lin % gridDim.x, lin / gridDim.x);
}

// 4-bit codes two to a byte (code 2b low nibble, code 2b+1 high nibble, two's complement) -> one int8
// each: what the integer g_w product multiplies when the activation was stored as int4 (Sec. 6.1).
// A lane turns 16 bytes into 32.
__global__ __launch_bounds__(256) void k_unpack_nibbles(const uint4 *__restrict__ in, uint4 *__restrict__ out, int64_t n16)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 x = in[i];
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
    uint32_t o[8];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = w[d] & 0x0F0F0F0Fu, hi = (w[d] >> 4) & 0x0F0F0F0Fu;
        // bytes (lo0, hi0, lo1, hi1) and (lo2, hi2, lo3, hi3): v_perm selectors 0-3 = second operand, 4-7 = first
        uint32_t a = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
        uint32_t b = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
        // sign-extend every byte's nibble: a set bit 3 fills the upper half of its byte
        a |= ((a >> 3) & 0x01010101u) * 0xF0u;
        b |= ((b >> 3) & 0x01010101u) * 0xF0u;
        o[2 * d] = a;
        o[2 * d + 1] = b;
    }
    out[2 * i] = make_uint4(o[0], o[1], o[2], o[3]);
    out[2 * i + 1] = make_uint4(o[4], o[5], o[6], o[7]);
}

hipError_t launch_unpack_nibbles(const void *in, int8_t *out, int64_t bytes_in, hipStream_t st)
{
    const int64_t n16 = bytes_in / 16;
    if (n16 <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_unpack_nibbles, dim3(static_cast<unsigned>((n16 + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint4 *>(in), reinterpret_cast<uint4 *>(out), n16);
    return hipGetLastError();
}

size_t hla_quant_ws_bytes(int64_t D) { return (static_cast<size_t>(D) * 4 + 255) & ~static_cast<size_t>(255); }

template <typename Tin, int B, int BASIS>
static hipError_t launch_hla_quant_t(const void *T, int64_t N, int D, int r, uint32_t k0, uint32_t k1, bool mant,
                                     int8_t *TqT, float *sT, float *coeffT, void *ws, hipStream_t st, bool p4 = false)
{
    constexpr int CPL = 128 / B;
    const int64_t nblk = N / B;
    uint32_t *amax = static_cast<uint32_t *>(ws);
    const Tin *t = static_cast<const Tin *>(T);
    dim3 grid(hla_grid_x(D, B), hla_grid_y(N, B));
    hipLaunchKernelGGL(k_hla_fill_u32, dim3((D + 255) / 256), dim3(256), 0, st, amax, D, 0u);
    hipLaunchKernelGGL((k_hla_absmax<Tin, B, BASIS>), grid, dim3(256), 0, st, t, N, D, r, amax);
    if (p4)   // the 4-bit store rounds by the seeded stream only
        hipLaunchKernelGGL((k_hla_quantize<Tin, B, BASIS, false, true>), grid, dim3(256), 0, st, t, N, D, r, amax, k0, k1, TqT, sT, coeffT);
    else if (mant)
        hipLaunchKernelGGL((k_hla_quantize<Tin, B, BASIS, true>), grid, dim3(256), 0, st, t, N, D, r, amax, k0, k1, TqT, sT, coeffT);
    else
        hipLaunchKernelGGL((k_hla_quantize<Tin, B, BASIS, false>), grid, dim3(256), 0, st, t, N, D, r, amax, k0, k1, TqT, sT, coeffT);
    return hipGetLastError();
}

hipError_t launch_hla_quant(const void *T, int64_t N, int D, int B, int r, int basis, bool is_f32, uint32_t k0,
                            uint32_t k1, bool mant, int8_t *TqT, float *sT, float *coeffT, void *ws, hipStream_t st, bool p4)
{
#define HLQ_HLAQ_CASE(BB)                                                                                  \
    case BB:                                                                                               \
        if (basis)                                                                                         \
            return is_f32 ? launch_hla_quant_t<float, BB, 1>(T, N, D, r, k0, k1, mant, TqT, sT, coeffT, ws, st, p4)  \
                          : launch_hla_quant_t<bf16_t, BB, 1>(T, N, D, r, k0, k1, mant, TqT, sT, coeffT, ws, st, p4); \
        return is_f32 ? launch_hla_quant_t<float, BB, 0>(T, N, D, r, k0, k1, mant, TqT, sT, coeffT, ws, st, p4)      \
                      : launch_hla_quant_t<bf16_t, BB, 0>(T, N, D, r, k0, k1, mant, TqT, sT, coeffT, ws, st, p4);
    switch (B) {
        HLQ_HLAQ_CASE(16)
        HLQ_HLAQ_CASE(32)
        HLQ_HLAQ_CASE(64)
    }
#undef HLQ_HLAQ_CASE
    return hipErrorInvalidValue;
}

// ---- the same three kernels on the column matrix of a channels-last image (Sec. 3.1), read through
// ---- ConvRows: the column matrix [N = Nb*Ho*Wo, D = kh*kw*C] is never stored ----------------------
template <typename Tin, int B, int BASIS>
__global__ __launch_bounds__(256) void k_hla_conv(const Tin *__restrict__ X, ConvShape g, int D, int r,
                                                  bf16_t *__restrict__ ThatT, float *__restrict__ coeffT)
{
    hla_body_src<B, BASIS>(ConvRows<Tin>{X, g}, g.N, D, r, ThatT, coeffT, blockIdx.x, blockIdx.y);
}

template <typename Tin, int B, int BASIS>
__global__ __launch_bounds__(256) void k_hla_absmax_conv(const Tin *__restrict__ X, ConvShape g, int D, int r,
                                                         uint32_t *__restrict__ amax_bits)
{
    hla_absmax_body_src<B, BASIS>(ConvRows<Tin>{X, g}, g.N, D, r, amax_bits, blockIdx.x, blockIdx.y);
}

template <typename Tin, int B, int BASIS, bool MANT>
__global__ __launch_bounds__(256) void k_hla_quantize_conv(const Tin *__restrict__ X, ConvShape g, int D, int r,
                                                           const uint32_t *__restrict__ amax_bits, uint32_t k0,
                                                           uint32_t k1, int8_t *__restrict__ TqT, float *__restrict__ sT,
                                                           float *__restrict__ coeffT)
{
    const int lin = reverse_same_xcd(blockIdx.x + blockIdx.y * gridDim.x, gridDim.x * gridDim.y,   // backwards, as above
                                     g.N * D * static_cast<int64_t>(sizeof(Tin)));
    hla_quantize_body_src<B, BASIS, MANT>(ConvRows<Tin>{X, g}, g.N, D, r, amax_bits, k0, k1, TqT, sT, coeffT, lin % gridDim.x,
                                          lin / gridDim.x);
}

bool hla_conv_ok(const ConvShape &g, int B) { return g.C % (128 / B) == 0; }

template <typename Tin, int B, int BASIS>
static hipError_t launch_hla_conv_t(const void *X, const ConvShape &g, int r, bf16_t *ThatT, float *coeffT, hipStream_t st)
{
    constexpr int CPL = 128 / B;
    const int D = g.kh * g.kw * g.C;
    dim3 grid(hla_grid_x(D, B), hla_grid_y(g.N, B));
    hipLaunchKernelGGL((k_hla_conv<Tin, B, BASIS>), grid, dim3(256), 0, st, static_cast<const Tin *>(X), g, D, r, ThatT, coeffT);
    return hipGetLastError();
}

hipError_t launch_hla_conv(const void *X, const ConvShape &g, int B, int r, int basis, bool is_f32, uint16_t *ThatT,
                           float *coeffT, hipStream_t st)
{
    if (!hla_conv_ok(g, B)) return hipErrorInvalidValue;
#define HLQ_HLAC_CASE(BB)                                                                        \
    case BB:                                                                                     \
        if (basis)                                                                               \
            return is_f32 ? launch_hla_conv_t<float, BB, 1>(X, g, r, ThatT, coeffT, st)          \
                          : launch_hla_conv_t<bf16_t, BB, 1>(X, g, r, ThatT, coeffT, st);        \
        return is_f32 ? launch_hla_conv_t<float, BB, 0>(X, g, r, ThatT, coeffT, st)              \
                      : launch_hla_conv_t<bf16_t, BB, 0>(X, g, r, ThatT, coeffT, st);
    switch (B) {
        HLQ_HLAC_CASE(16)
        HLQ_HLAC_CASE(32)
        HLQ_HLAC_CASE(64)
    }
#undef HLQ_HLAC_CASE
    return hipErrorInvalidValue;
}

template <typename Tin, int B, int BASIS>
static hipError_t launch_hla_quant_conv_t(const void *X, const ConvShape &g, int r, uint32_t k0, uint32_t k1, bool mant,
                                          int8_t *TqT, float *sT, float *coeffT, void *ws, hipStream_t st)
{
    constexpr int CPL = 128 / B;
    const int D = g.kh * g.kw * g.C;
    uint32_t *amax = static_cast<uint32_t *>(ws);
    const Tin *x = static_cast<const Tin *>(X);
    dim3 grid(hla_grid_x(D, B), hla_grid_y(g.N, B));
    hipLaunchKernelGGL(k_hla_fill_u32, dim3((D + 255) / 256), dim3(256), 0, st, amax, D, 0u);
    hipLaunchKernelGGL((k_hla_absmax_conv<Tin, B, BASIS>), grid, dim3(256), 0, st, x, g, D, r, amax);
    if (mant)
        hipLaunchKernelGGL((k_hla_quantize_conv<Tin, B, BASIS, true>), grid, dim3(256), 0, st, x, g, D, r, amax, k0, k1, TqT, sT, coeffT);
    else
        hipLaunchKernelGGL((k_hla_quantize_conv<Tin, B, BASIS, false>), grid, dim3(256), 0, st, x, g, D, r, amax, k0, k1, TqT, sT, coeffT);
    return hipGetLastError();
}

hipError_t launch_hla_quant_conv(const void *X, const ConvShape &g, int B, int r, int basis, bool is_f32, uint32_t k0,
                                 uint32_t k1, bool mant, int8_t *TqT, float *sT, float *coeffT, void *ws, hipStream_t st)
{
    if (!hla_conv_ok(g, B)) return hipErrorInvalidValue;
#define HLQ_HLAQC_CASE(BB)                                                                                     \
    case BB:                                                                                                   \
        if (basis)                                                                                             \
            return is_f32 ? launch_hla_quant_conv_t<float, BB, 1>(X, g, r, k0, k1, mant, TqT, sT, coeffT, ws, st)  \
                          : launch_hla_quant_conv_t<bf16_t, BB, 1>(X, g, r, k0, k1, mant, TqT, sT, coeffT, ws, st); \
        return is_f32 ? launch_hla_quant_conv_t<float, BB, 0>(X, g, r, k0, k1, mant, TqT, sT, coeffT, ws, st)      \
                      : launch_hla_quant_conv_t<bf16_t, BB, 0>(X, g, r, k0, k1, mant, TqT, sT, coeffT, ws, st);
    switch (B) {
        HLQ_HLAQC_CASE(16)
        HLQ_HLAQC_CASE(32)
        HLQ_HLAQC_CASE(64)
    }
#undef HLQ_HLAQC_CASE
    return hipErrorInvalidValue;
}

}  // namespace hlq
