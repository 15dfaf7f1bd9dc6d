// Convolution layers (arXiv 2406.15102, Sec. 3.1): a convolution is the linear layer's product
// with the spatial positions as the sequence, so its backward pass is the same two stage lists on
// the column matrix of the input.  This file holds the two pieces of glue around them, for
// channels-last tensors:
//   column matrix   x [Nb, H, W, C] -> cols [Nb*Ho*Wo, kh*kw*C]; row t = (n, ho, wo) is the receptive
//                   field of output position (ho, wo), columns ordered (ky, kx, c) like the trailing
//                   axes of a channels-last weight [O, kh, kw, C]; taps outside the image read 0;
//   fold            its adjoint: pixel (n, h, w, c) of the image gradient is the sum of every
//                   entry of the column gradient that was copied from it, added in fp32 in
//                   ascending (ky, kx) order (deterministic), rounded once to the output type.
// Both are plain HBM-bound data movement in 16-byte units (8 bf16 / 4 fp32 channels) when the channel
// count allows, else element by element.  The column matrix gives a wavefront one row of its output
// (one receptive field): the row index is decomposed once per wavefront and a lane spends two integer
// divisions per unit.  The fold gives a lane one unit of the image and a wavefront 64 units of one
// image row, so that even small feature maps make thousands of wavefronts.
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"
#include "reduce_body.hpp"

namespace hlq {

template <int VB> struct Unit;
template <> struct Unit<16> { typedef uint4 type; };
template <> struct Unit<4> { typedef uint32_t type; };
template <> struct Unit<2> { typedef uint16_t type; };

// Cu = channels in units of VB bytes
template <int VB>
__global__ __launch_bounds__(256) void k_im2col(const void *__restrict__ X, ConvShape g, int Cu, void *__restrict__ cols)
{
    typedef typename Unit<VB>::type U;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (t >= g.N) return;
    const int lane = threadIdx.x & 63;
    const int wo = static_cast<int>(t % g.Wo);
    const int64_t t2 = t / g.Wo;
    const int ho = static_cast<int>(t2 % g.Ho);
    const int64_t n = t2 / g.Ho;
    const int h0 = ho * g.sh - g.ph, w0 = wo * g.sw - g.pw;
    const U *x = static_cast<const U *>(X) + n * g.H * g.W * Cu;
    const int row_units = g.kh * g.kw * Cu;
    U *out = static_cast<U *>(cols) + t * row_units;
    for (int v = lane; v < row_units; v += 64) {
        const int tap = v / Cu, cu = v - tap * Cu;
        const int ky = tap / g.kw, kx = tap - ky * g.kw;
        const int hi = h0 + ky * g.dh, wi = w0 + kx * g.dw;
        U val = {};
        if (hi >= 0 && hi < g.H && wi >= 0 && wi < g.W) val = x[(static_cast<int64_t>(hi) * g.W + wi) * Cu + cu];
        out[v] = val;
    }
}

template <typename T> struct Chan;
template <> struct Chan<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void add(const bf16_t *p, float *s)
    {
        const uint4 q = *reinterpret_cast<const uint4 *>(p);
        s[0] += bf16_lo(q.x); s[1] += bf16_hi(q.x); s[2] += bf16_lo(q.y); s[3] += bf16_hi(q.y);
        s[4] += bf16_lo(q.z); s[5] += bf16_hi(q.z); s[6] += bf16_lo(q.w); s[7] += bf16_hi(q.w);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float *s)
    {
        uint4 q = {pack_bf16(s[0], s[1]), pack_bf16(s[2], s[3]), pack_bf16(s[4], s[5]), pack_bf16(s[6], s[7])};
        *reinterpret_cast<uint4 *>(p) = q;
    }
    static __device__ __forceinline__ float load1(const bf16_t *p) { return bf16_lo(*p); }
    static __device__ __forceinline__ void store1(bf16_t *p, float s) { *p = static_cast<bf16_t>(pack_bf16(s, 0.0f) & 0xFFFFu); }
};
template <> struct Chan<float> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void add(const float *p, float *s)
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        s[0] += q.x; s[1] += q.y; s[2] += q.z; s[3] += q.w;
    }
    static __device__ __forceinline__ void store(float *p, const float *s)
    {
        *reinterpret_cast<float4 *>(p) = make_float4(s[0], s[1], s[2], s[3]);
    }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
    static __device__ __forceinline__ void store1(float *p, float s) { *p = s; }
};

// One lane per pixel and group of VEC channels (Chan<T>::VEC, or 1); a wavefront covers 64 such
// units of one image row (n, h), so the row's decomposition and the vertical taps are wave-uniform.
// KS > 0: kh = kw = KS known at compile time -- the tap loop unrolls and its loads are in flight
// together.  A tap that no output position pairs with this pixel loads from row 0 of the column
// matrix instead (always inside the tensor) and is not added.
template <typename T, bool VECTOR, int KS>
__global__ __launch_bounds__(256) void k_col2im(const T *__restrict__ cols, ConvShape g, int chunks, T *__restrict__ dx,
                                                SplitReduce red)
{
    constexpr int VEC = VECTOR ? Chan<T>::VEC : 1;
    // a side job that shares the launch: the split-K reduction of the weight gradient's product
    if (blockIdx.x < static_cast<unsigned>(red.blocks)) {
        splitk_reduce_job(red, blockIdx.x);
        return;
    }
    const int64_t wid = static_cast<int64_t>(blockIdx.x - red.blocks) * 4 + (threadIdx.x >> 6);
    const int64_t rowi = wid / chunks;
    if (rowi >= static_cast<int64_t>(g.Nb) * g.H) return;
    const int chunk = static_cast<int>(wid - rowi * chunks);
    const int h = static_cast<int>(rowi % g.H);
    const int64_t n = rowi / g.H;
    const int Cv = g.C / VEC;
    const int v = chunk * 64 + (threadIdx.x & 63);
    if (v >= g.W * Cv) return;
    const int w = v / Cv, c = (v - w * Cv) * VEC;
    const int KH = KS ? KS : g.kh, KW = KS ? KS : g.kw;
    const int64_t I = static_cast<int64_t>(KH) * KW * g.C;
    float s[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) s[k] = 0.0f;
    // constant trip counts (KS > 0) unroll by themselves; the general case stays a loop
    for (int ky = 0; ky < KH; ++ky) {
        const int hn = h + g.ph - ky * g.dh;              // = ho * stride for the output row that read this pixel
        const int ho = g.sh == 1 ? hn : hn / g.sh;
        const bool okh = hn >= 0 && ho * g.sh == hn && ho < g.Ho;
        for (int kx = 0; kx < KW; ++kx) {
            const int wn = w + g.pw - kx * g.dw;
            const int wo = g.sw == 1 ? wn : wn / g.sw;
            const bool ok = okh && wn >= 0 && wo * g.sw == wn && wo < g.Wo;
            const int64_t t = ok ? (n * g.Ho + ho) * g.Wo + wo : 0;
            const T *p = cols + t * I + (ky * KW + kx) * g.C + c;
            float a[VEC];
#pragma unroll
            for (int k = 0; k < VEC; ++k) a[k] = 0.0f;
            if (VECTOR) Chan<T>::add(p, a);
            else a[0] = Chan<T>::load1(p);
            if (ok) {
#pragma unroll
                for (int k = 0; k < VEC; ++k) s[k] += a[k];
            }
        }
    }
    T *o = dx + ((n * g.H + h) * g.W + w) * g.C + c;
    if (VECTOR) Chan<T>::store(o, s);
    else Chan<T>::store1(o, s[0]);
}

hipError_t launch_im2col(const void *X, const ConvShape &g, bool is_f32, void *cols, hipStream_t st)
{
    const int e = is_f32 ? 4 : 2;
    const unsigned grid = static_cast<unsigned>((g.N + 3) / 4);
    if ((g.C * e) % 16 == 0) hipLaunchKernelGGL(k_im2col<16>, dim3(grid), dim3(256), 0, st, X, g, g.C * e / 16, cols);
    else if (is_f32) hipLaunchKernelGGL(k_im2col<4>, dim3(grid), dim3(256), 0, st, X, g, g.C, cols);
    else hipLaunchKernelGGL(k_im2col<2>, dim3(grid), dim3(256), 0, st, X, g, g.C, cols);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_col2im_t(const void *cols, const ConvShape &g, void *dx, hipStream_t st, const SplitReduce &red)
{
    const T *c = static_cast<const T *>(cols);
    T *o = static_cast<T *>(dx);
    const bool vec = g.C % Chan<T>::VEC == 0;
    const int chunks = (g.W * (vec ? g.C / Chan<T>::VEC : g.C) + 63) / 64;
    const int64_t waves = static_cast<int64_t>(g.Nb) * g.H * chunks;
    if (waves + 3 >= (int64_t(1) << 33) || red.blocks < 0 || red.blocks > (1 << 28)) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>((waves + 3) / 4 + red.blocks));
    const bool k3 = g.kh == 3 && g.kw == 3;
    if (vec) {
        if (k3) hipLaunchKernelGGL((k_col2im<T, true, 3>), grid, dim3(256), 0, st, c, g, chunks, o, red);
        else hipLaunchKernelGGL((k_col2im<T, true, 0>), grid, dim3(256), 0, st, c, g, chunks, o, red);
    } else {
        if (k3) hipLaunchKernelGGL((k_col2im<T, false, 3>), grid, dim3(256), 0, st, c, g, chunks, o, red);
        else hipLaunchKernelGGL((k_col2im<T, false, 0>), grid, dim3(256), 0, st, c, g, chunks, o, red);
    }
    return hipGetLastError();
}

hipError_t launch_col2im(const void *cols, const ConvShape &g, bool is_f32, void *dx, hipStream_t st, const SplitReduce *red)
{
    const SplitReduce none{};
    const SplitReduce &job = red ? *red : none;
    return is_f32 ? launch_col2im_t<float>(cols, g, dx, st, job) : launch_col2im_t<bf16_t>(cols, g, dx, st, job);
}

}  // namespace hlq
