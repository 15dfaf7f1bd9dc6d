// Device-side building blocks shared by the gfx950 kernels: element loads, the in-register
// fast Walsh-Hadamard transform, the stochastic-rounding random stream and the 4-bit quantiser.
//
// Numerical contract (arXiv 2406.15102, Sec. 3.2 / 5.1 / 6.1, as fixed by this library):
//   * H is the +-1 natural-order Walsh-Hadamard matrix; a coefficient is the sum of its B signed
//     terms added pairwise in index order.  A radix-2 butterfly network with strides 1, 2, 4, ...
//     (ascending) evaluates exactly that expression tree, so the stage order below is fixed.
//   * code = clamp(floor(fma(x, 7/absmax, (byte + 0.5)/256)), -7, 7), byte taken from word
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

// One butterfly stage between lanes l and l^MASK (MASK in {1, 2, 4}): the lane with the bit
// clear keeps a+b, the other a-b, a being the value of the lower lane.
template <int MASK>
__device__ __forceinline__ float lane_xor(float x)
{
    int xi = __builtin_bit_cast(int, x);
    int r;
    if (MASK == 1) r = __builtin_amdgcn_update_dpp(0, xi, 0xB1, 0xF, 0xF, true);       // quad_perm [1,0,3,2]
    else if (MASK == 2) r = __builtin_amdgcn_update_dpp(0, xi, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    else r = __builtin_amdgcn_ds_swizzle(xi, 0x101F);                                  // lane ^ 4
    return __builtin_bit_cast(float, r);
}

template <int MASK>
__device__ __forceinline__ float butterfly_lanes(float x, bool upper)
{
    float p = lane_xor<MASK>(x);
    float own = upper ? -x : x;
    return p + own;
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

// Four codes from four values and one random word, packed little-endian into a dword.
__device__ __forceinline__ int quant_code(float x, float inv, uint32_t byte)
{
    float u = (static_cast<float>(byte) + 0.5f) * 0.00390625f;
    float t = __builtin_fmaf(x, inv, u);
    int q = static_cast<int>(__builtin_floorf(t));
    q = q > 7 ? 7 : q;
    q = q < -7 ? -7 : q;
    return q;
}

__device__ __forceinline__ uint32_t quant_pack4(float x0, float x1, float x2, float x3, float inv, uint32_t w)
{
    uint32_t q0 = static_cast<uint32_t>(quant_code(x0, inv, w & 0xFFu)) & 0xFFu;
    uint32_t q1 = static_cast<uint32_t>(quant_code(x1, inv, (w >> 8) & 0xFFu)) & 0xFFu;
    uint32_t q2 = static_cast<uint32_t>(quant_code(x2, inv, (w >> 16) & 0xFFu)) & 0xFFu;
    uint32_t q3 = static_cast<uint32_t>(quant_code(x3, inv, w >> 24));
    return q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
}

__device__ __forceinline__ float absmax_to_inv(float a) { return a > 0.0f ? 7.0f / a : 0.0f; }
__device__ __forceinline__ float absmax_to_scale(float a) { return a / 7.0f; }

}  // namespace hlq
