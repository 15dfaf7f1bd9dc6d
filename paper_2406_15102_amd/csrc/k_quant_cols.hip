// K1T -- stages 3-4 of the g_x list (arXiv 2406.15102, Sec. 6.1): H_O^T . W, i.e. the block
// Hadamard transform (Sec. 3.2) over groups of B consecutive ROWS of W [d_out, d_in], then 4-bit
// stochastic quantisation (Sec. 5.1) with one absmax scale per in-feature (= per column of W,
// = per row of the transposed, reduction-contiguous output WqT [d_in, d_out]).
//
// A lane owns CPL = 128/B adjacent columns and B consecutive rows: B row loads (16 B per lane for
// bf16) put whole Hadamard blocks in its registers, so the transform needs no lane exchange.  A
// workgroup is B lanes side by side (runs of 256 B of a row) times 256/B consecutive row blocks,
// whose codes are neighbours in a row of the transposed output (runs of 256 bytes, 128 packed):
// thousands of independent workgroups even for one layer, and long runs both ways.
// The column absmax spans all of d_out, hence two passes over W (the second mostly served by the
// last-level cache when W fits there):
//   zero    amax[d_in] = 0
//   pass 1  transform, per-column max over the workgroup's rows (LDS), one atomic max per column
//           and workgroup.  max() is order-independent and the values are non-negative floats,
//           whose bit patterns order like unsigned integers: the result is deterministic.
//   pass 2  transform again, quantise, write B codes per column and row block.
#include "quant_cols_body.hpp"
#include "hlq_kernels.hpp"

#include <mutex>

namespace hlq {

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t *p, int n, uint32_t value)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = value;
}

template <typename Tin, int B>
__global__ __launch_bounds__(256) void k_cols_absmax(const Tin *__restrict__ W, int O, int I,
                                                     uint32_t *__restrict__ amax_bits)
{
    cols_absmax_body<Tin, B>(W, O, I, amax_bits, blockIdx.x, blockIdx.y);
}

template <typename Tin, int B, bool PACKED, bool MANT>
__global__ __launch_bounds__(256) void k_cols_quantize(const Tin *__restrict__ W, int O, int I,
                                                       const uint32_t *__restrict__ amax_bits, uint32_t k0, uint32_t k1,
                                                       float qmax, int8_t *__restrict__ WqT, float *__restrict__ sW,
                                                       float *__restrict__ coeffT)
{
    // backwards (reverse_same_xcd): what pass 1 read last is what the last-level cache still holds
    const int lin = reverse_same_xcd(blockIdx.x + blockIdx.y * gridDim.x, gridDim.x * gridDim.y,
                                     static_cast<int64_t>(O) * I * static_cast<int64_t>(sizeof(Tin)));
    cols_quantize_body<Tin, B, PACKED, MANT>(W, O, I, amax_bits, k0, k1, qmax, WqT, sW, coeffT, lin % gridDim.x, lin / gridDim.x);
}

size_t quant_cols_ws_bytes(int64_t /*O*/, int64_t I)
{
    // amax bit patterns, one uint32 per in-feature
    return (static_cast<size_t>(I) * 4 + 255) & ~static_cast<size_t>(255);
}

template <typename Tin, int B>
static hipError_t launch_cols_pass1_t(const void *W, int O, int I, void *ws, hipStream_t st)
{
    constexpr int CPL = 128 / B;
    uint32_t *amax = static_cast<uint32_t *>(ws);
    dim3 grid(cols_grid_x(I, B), cols_grid_y(O, B));
    hipLaunchKernelGGL(k_fill_u32, dim3((I + 255) / 256), dim3(256), 0, st, amax, I, 0u);
    hipLaunchKernelGGL((k_cols_absmax<Tin, B>), grid, dim3(256), 0, st, static_cast<const Tin *>(W), O, I, amax);
    return hipGetLastError();
}

template <typename Tin, int B>
static hipError_t launch_cols_pass2_t(const void *W, int O, int I, uint32_t k0, uint32_t k1, float qmax, bool packed,
                                      bool mant, int8_t *WqT, float *sW, float *coeffT, const void *ws, hipStream_t st)
{
    constexpr int CPL = 128 / B;
    const uint32_t *amax = static_cast<const uint32_t *>(ws);
    const Tin *w = static_cast<const Tin *>(W);
    dim3 grid(cols_grid_x(I, B), cols_grid_y(O, B));
#define HLQ_COLS2_LAUNCH(P, M) \
    hipLaunchKernelGGL((k_cols_quantize<Tin, B, P, M>), grid, dim3(256), 0, st, w, O, I, amax, k0, k1, qmax, WqT, sW, coeffT)
    if (packed) {
        if (mant) HLQ_COLS2_LAUNCH(true, true); else HLQ_COLS2_LAUNCH(true, false);
    } else {
        if (mant) HLQ_COLS2_LAUNCH(false, true); else HLQ_COLS2_LAUNCH(false, false);
    }
#undef HLQ_COLS2_LAUNCH
    return hipGetLastError();
}

hipError_t launch_quant_cols_pass2(const void *W, int O, int I, int B, bool is_f32, uint32_t k0, uint32_t k1,
                                   float qmax, bool packed, bool mant, int8_t *WqT, float *sW, float *coeffT,
                                   const void *ws, hipStream_t st)
{
#define HLQ_COLS2_CASE(BB)                                                                                               \
    case BB:                                                                                                             \
        return is_f32 ? launch_cols_pass2_t<float, BB>(W, O, I, k0, k1, qmax, packed, mant, WqT, sW, coeffT, ws, st)     \
                      : launch_cols_pass2_t<bf16_t, BB>(W, O, I, k0, k1, qmax, packed, mant, WqT, sW, coeffT, ws, st);
    switch (B) {
        HLQ_COLS2_CASE(16)
        HLQ_COLS2_CASE(32)
        HLQ_COLS2_CASE(64)
    }
#undef HLQ_COLS2_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_quant_cols(const void *W, int O, int I, int B, bool is_f32, uint32_t k0, uint32_t k1,
                             float qmax, bool packed, bool mant, int8_t *WqT, float *sW, float *coeffT, void *ws,
                             hipStream_t st)
{
    hipError_t e = hipErrorInvalidValue;
#define HLQ_COLS_CASE(BB)                                                                            \
    case BB:                                                                                         \
        e = is_f32 ? launch_cols_pass1_t<float, BB>(W, O, I, ws, st) : launch_cols_pass1_t<bf16_t, BB>(W, O, I, ws, st); \
        break;
    switch (B) {
        HLQ_COLS_CASE(16)
        HLQ_COLS_CASE(32)
        HLQ_COLS_CASE(64)
    }
#undef HLQ_COLS_CASE
    if (e != hipSuccess) return e;
    return launch_quant_cols_pass2(W, O, I, B, is_f32, k0, k1, qmax, packed, mant, WqT, sW, coeffT, ws, st);
}

// ---- scratch for callers that cannot allocate -------------------------------------------------
// The column maxima of launch_quant_cols in device memory that belongs to the code object: one
// copy per GPU the library runs on, held until the process ends.  On the host the array's name is
// only a handle: its device address is asked for once per device and kept.
static __device__ __align__(256) __attribute__((used)) uint32_t scratch[kQuantColsStaticMaxI];

hipError_t quant_cols_static_scratch(void **ptr)
{
    static std::mutex mtx;
    static void *addr[64] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mtx);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return hipSuccess;
}

}  // namespace hlq
