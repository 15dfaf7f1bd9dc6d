// Device-side building blocks shared by the gfx950 kernels: element loads, the in-register
// fast Walsh-Hadamard transform, the stochastic-rounding random stream and the 4-bit quantiser.
//
// Numerical contract (arXiv 2406.15102, Sec. 3.2 / 5.1 / 6.1, as fixed by this library):
//   * H is the +-1 natural-order Walsh-Hadamard matrix; a coefficient is the sum of its B signed
//     terms added pairwise in index order.  A radix-2 butterfly network with strides 1, 2, 4, ...
//     (ascending) evaluates exactly that expression tree, so the stage order below is fixed.
//   * code = floor(fma(x, qmax/absmax, (byte + 0.5)/256)) (always inside [-qmax, qmax]; qmax = 7
//     or 127), byte taken from word
//     number row*(K/4) + pos/4 of a keyed counter stream, byte pos%4 of that word.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hlq {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));

// Two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    v2f p = {lo, hi};
    v2bf q = __builtin_convertvector(p, v2bf);
    return __builtin_bit_cast(uint32_t, q);
}

// ---- element loads: NE consecutive elements widened to fp32 --------------------------------
template <typename T, int NE> struct Loader;

template <> struct Loader<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t *p, float *v)
    {
        uint4 w = *reinterpret_cast<const uint4 *>(p);
        v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x); v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
        v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z); v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
    }
};
template <> struct Loader<bf16_t, 4> {
    static __device__ __forceinline__ void load(const bf16_t *p, float *v)
    {
        uint2 w = *reinterpret_cast<const uint2 *>(p);
        v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x); v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
    }
};
template <> struct Loader<bf16_t, 2> {
    static __device__ __forceinline__ void load(const bf16_t *p, float *v)
    {
        uint32_t w = *reinterpret_cast<const uint32_t *>(p);
        v[0] = bf16_lo(w); v[1] = bf16_hi(w);
    }
};
template <> struct Loader<float, 8> {
    static __device__ __forceinline__ void load(const float *p, float *v)
    {
        float4 a = *reinterpret_cast<const float4 *>(p);
        float4 b = *reinterpret_cast<const float4 *>(p + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};
template <> struct Loader<float, 4> {
    static __device__ __forceinline__ void load(const float *p, float *v)
    {
        float4 a = *reinterpret_cast<const float4 *>(p);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    }
};
template <> struct Loader<float, 2> {
    static __device__ __forceinline__ void load(const float *p, float *v)
    {
        float2 a = *reinterpret_cast<const float2 *>(p);
        v[0] = a.x; v[1] = a.y;
    }
};

// Workgroup `lin` of `total`, counted from the other end but on the same XCD (workgroups go to the eight XCDs
// round-robin, index mod 8): the second pass over a tensor walks it backwards, so that it starts on what the
// first pass read last -- what the last-level cache still holds of a tensor larger than it -- and a workgroup
// still finds in its own XCD's L2 what its counterpart of the first pass left there.
// Only for tensors of more than half that cache (`bytes`): a smaller one is found there whole, and in order it
// measured a little better (4096 x 4096 activation, int8 store: 16.6 us against 17.5 backwards).
constexpr int64_t kReverseSecondPassBytes = int64_t(128) << 20;
__device__ __forceinline__ int reverse_same_xcd(int lin, int total, int64_t bytes)
{
    const int n8 = total & ~7;
    return (bytes > kReverseSecondPassBytes && lin < n8) ? (n8 - 8 - (lin & ~7)) + (lin & 7) : lin;
}

// ---- in-register FWHT over v[0..n), element stride `es` in the array, strides ascending -----
template <int NPT, int ES>
__device__ __forceinline__ void fwht_regs(float *v)
{
#pragma unroll
    for (int h = 1; h < NPT; h *= 2) {
#pragma unroll
        for (int base = 0; base < NPT; base += 2 * h) {
#pragma unroll
            for (int k = base; k < base + h; ++k) {
                float a = v[k * ES], b = v[(k + h) * ES];
                v[k * ES] = a + b;
                v[(k + h) * ES] = a - b;
            }
        }
    }
}

// One butterfly stage between lanes l and l^MASK (MASK in {1, 2, 4}) in ONE instruction where the
// exchange is a DPP quad permute: x <- partner * sigma + x with sigma = +1 in the lane whose MASK
// bit is clear and -1 in the other.  The product is exact, so the single rounding is that of the
// add/subtract of the butterfly.  The lower lane gets a + b; the upper lane gets b - a, i.e. the
// NEGATIVE of the butterfly's difference a - b... with a = lower lane's value: upper holds
// x_upper - x_lower = -(a - b).  Callers carry that sign per lane (it is the same for both lanes of
// every later exchange, because they differ in a higher lane bit only) and fold it into whatever
// consumes the value.  The s_nop covers the VALU-write -> DPP-read hazard, which the compiler
// cannot see inside an asm statement.
template <int MASK>
__device__ __forceinline__ float butterfly_lanes_signed(float x, float sigma)
{
    if (MASK == 1) {
        asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "+v"(x) : "v"(x), "v"(sigma));
        return x;
    } else if (MASK == 2) {
        asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "+v"(x) : "v"(x), "v"(sigma));
        return x;
    } else {
        const float p = __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, x), 0x101F));  // lane ^ 4
        return __builtin_fmaf(p, sigma, x);
    }
}

// Row of the natural-order Hadamard matrix kept as coefficient k of the low-rank projection.
// BASIS 0: row k.  BASIS 1: the row with k sign changes (sequency order), which is the
// bit-reversed Gray code of k.  Constant-folds when k is a compile-time constant.
template <int B, int BASIS>
__host__ __device__ constexpr int kept_row(int k)
{
    if (BASIS == 0) return k;
    const int g = k ^ (k >> 1);
    int n = 0;
    for (int lo = 1, hi = B >> 1; lo < B; lo <<= 1, hi >>= 1)
        if (g & lo) n |= hi;
    return n;
}

// ---- random stream ---------------------------------------------------------------------------
// Word `counter` of the stream keyed by (k0, k1): a keyed xorshift-multiply bijection of the
// counter (multipliers of the public-domain "lowbias32" integer hash).
__device__ __forceinline__ uint32_t rand_word(uint32_t counter, uint32_t k0, uint32_t k1)
{
    uint32_t x = counter ^ k0;
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x ^= k1;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

// floor(t) as an integer in one instruction (v_cvt_flr_i32_f32).
__device__ __forceinline__ int floor_to_int(float t)
{
    int r;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(t));
    return r;
}

// One code: floor(fma(x, inv, u)), u = (byte + 0.5) / 256 (exact in fp32, built with one fma).
// No clamp is needed: |x| <= absmax and inv = RN(qmax / absmax) give |x*inv| <= qmax (1 + 2^-24),
// and u lies in [2^-9, 1 - 2^-9], so the rounded sum stays inside (-qmax, qmax + 1) and its floor
// inside [-qmax, qmax] (a zero row has inv = 0 and floor(u) = 0).  Inf/NaN inputs are outside the
// contract.
__device__ __forceinline__ int quant_code(float x, float inv, float byte_as_float)
{
    const float u = __builtin_fmaf(byte_as_float, 0.00390625f, 0.001953125f);
    return floor_to_int(__builtin_fmaf(x, inv, u));
}

// Four codes from four values and one random word, packed little-endian into a dword
// (two's-complement bytes, as the int8 MFMA reads them).
__device__ __forceinline__ uint32_t quant_pack4(float x0, float x1, float x2, float x3, float inv, uint32_t w)
{
    const uint32_t q0 = static_cast<uint32_t>(quant_code(x0, inv, static_cast<float>(w & 0xFFu)));
    const uint32_t q1 = static_cast<uint32_t>(quant_code(x1, inv, static_cast<float>((w >> 8) & 0xFFu)));
    const uint32_t q2 = static_cast<uint32_t>(quant_code(x2, inv, static_cast<float>((w >> 16) & 0xFFu)));
    const uint32_t q3 = static_cast<uint32_t>(quant_code(x3, inv, static_cast<float>(w >> 24)));
    // v_perm_b32: selector bytes 0-3 pick bytes of the second operand, 4-7 of the first, 0x0c = zero
    const uint32_t lo = __builtin_amdgcn_perm(q1, q0, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(q3, q2, 0x04000c0cu);
    return lo | hi;
}

// The paper's pseudo-stochastic rounding (Sec. 6.1): the low 11 bits of the value's own binary32
// pattern replace the random number, u = (m + 0.5) / 2048 (exact, one fma).  A sign flip of the
// value (see butterfly_lanes_signed) leaves those bits alone.
__device__ __forceinline__ int quant_code_mantissa(float x, float inv)
{
    const float m = static_cast<float>(__float_as_uint(x) & 0x7FFu);
    const float u = __builtin_fmaf(m, 0.00048828125f, 0.000244140625f);
    return floor_to_int(__builtin_fmaf(x, inv, u));
}

// Four codes packed into a dword, rounding by the seeded stream (word `counter` of the stream keyed
// by k0, k1) or, with MANT, by the values' own low mantissa bits.
template <bool MANT>
__device__ __forceinline__ uint32_t quant_pack4r(float x0, float x1, float x2, float x3, float inv, uint32_t counter,
                                                 uint32_t k0, uint32_t k1)
{
    if (!MANT) return quant_pack4(x0, x1, x2, x3, inv, rand_word(counter, k0, k1));
    const uint32_t q0 = static_cast<uint32_t>(quant_code_mantissa(x0, inv));
    const uint32_t q1 = static_cast<uint32_t>(quant_code_mantissa(x1, inv));
    const uint32_t q2 = static_cast<uint32_t>(quant_code_mantissa(x2, inv));
    const uint32_t q3 = static_cast<uint32_t>(quant_code_mantissa(x3, inv));
    return __builtin_amdgcn_perm(q1, q0, 0x0c0c0400u) | __builtin_amdgcn_perm(q3, q2, 0x04000c0cu);
}

// Eight 4-bit codes from two dwords of int8 codes (as quant_pack4 makes them), two to a byte:
// code 2b in the low nibble of byte b, code 2b+1 in the high nibble, two's complement.
__device__ __forceinline__ uint32_t nibble_pack8(uint32_t lo, uint32_t hi)
{
    // bytes (c0, c1, c2, c3) -> bits 0..7 = c0 | c1 << 4, bits 16..23 = c2 | c3 << 4
    const uint32_t a = ((lo >> 4) & 0x00F000F0u) | (lo & 0x000F000Fu);
    const uint32_t b = ((hi >> 4) & 0x00F000F0u) | (hi & 0x000F000Fu);
    return __builtin_amdgcn_perm(b, a, 0x06040200u);   // bytes 0, 2 of a, then bytes 0, 2 of b
}

// qmax = 7 for 4-bit codes, 127 for 8-bit codes (int8 warm-up phase, integer g_w path).
__device__ __forceinline__ float absmax_to_inv(float a, float qmax) { return a > 0.0f ? qmax / a : 0.0f; }
__device__ __forceinline__ float absmax_to_scale(float a, float qmax) { return a / qmax; }

}  // namespace hlq
