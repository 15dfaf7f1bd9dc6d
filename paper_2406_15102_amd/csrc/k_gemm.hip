// K2 / K4 -- the two matrix products of the HLQ backward pass (arXiv 2406.15102, Sec. 6.1):
//   K2  stage 5-6 of the g_x list: int8 x int8 -> int32 product of the 4-bit codes (exact), then
//       dequantisation by the two per-row scales and 1/B            (v_mfma_i32_32x32x32_i8)
//   K4  stage 5 of the g_w list: bf16 product over the compressed token axis, fp32 accumulation,
//       scaled by 1/B                                               (v_mfma_f32_32x32x16_bf16)
// Both are "NT" products C[m,n] = sum_k A[m,k] Bm[n,k] with the reduction axis contiguous in both
// operands, and both MFMA shapes consume 16 B per lane and operand for a 32-byte slice of k, so one
// kernel template written in bytes serves the two.
//
// Tiling: a workgroup of 4 wavefronts (2 x 2) owns a (64*WM) x (64*WN) tile of C; each wavefront
// a (32*WM) x (32*WN) sub-tile held as WM x WN MFMA accumulators.  k advances 64 B per step through
// a double-buffered LDS tile; global loads for step t+1 are issued before the MFMAs of step t.
// LDS rows are 64 B (four 16-B chunks) with the chunk index xor-swizzled by the row so that the
// ds_read_b128 of 32 consecutive rows and the ds_write_b128 of the staging pass spread over all banks.
// The MFMA's A operand is fed from Bm and its B operand from A, which leaves each lane with four
// consecutive n for one m: C is written in 8- or 16-byte pieces.
// Workgroup ids are remapped so that each XCD (ids congruent mod 8) works on a compact patch of
// tiles and re-uses operand rows in its own L2.
#include "hlq_device.hpp"
#include "hlq_kernels.hpp"

namespace hlq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 16-B chunk (a first-class vector: stays in registers)
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int KIND> struct Mma;
template <> struct Mma<0> {
    typedef v16i acc_t;
    static __device__ __forceinline__ acc_t zero() { acc_t z = {0}; return z; }
    static __device__ __forceinline__ acc_t mma(const u32x4 &x, const u32x4 &y, acc_t c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(v4i, x), __builtin_bit_cast(v4i, y), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(int v) { return static_cast<float>(v); }
};
template <> struct Mma<1> {
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t zero() { acc_t z = {0.0f}; return z; }
    static __device__ __forceinline__ acc_t mma(const u32x4 &x, const u32x4 &y, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x), __builtin_bit_cast(v8bf, y), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_float(float v) { return v; }
};

struct GemmDev {
    const char *A;
    const char *Bm;
    int M, N;
    int Kb;            // bytes per operand row
    const float *sA;
    const float *sB;
    float alpha;
    void *C;
    int c_is_f32;
    int32_t *acc;
    int tiles_m, tiles_n;
};

// position of 16-B chunk c of LDS row `row` (4 chunks per row)
__device__ __forceinline__ int lds_chunk(int row, int c)
{
    const int f = (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
    return row * 4 + (c ^ f);
}

template <int KIND, int WM, int WN>
__global__ __launch_bounds__(256) void k_gemm_nt(GemmDev g)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int GROUP = 4;
    __shared__ u32x4 lds[2][(BM + BN) * 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;

    // ---- workgroup id -> tile, XCD-aware ----
    int tm, tn;
    {
        const int nb = g.tiles_m * g.tiles_n;
        const int pid = blockIdx.x;
        const int xcd = pid & 7, idx = pid >> 3;
        const int per = nb >> 3, rem = nb & 7;
        const int logical = xcd * per + (xcd < rem ? xcd : rem) + idx;
        const int width = GROUP * g.tiles_n;
        const int group = logical / width;
        const int first_m = group * GROUP;
        const int gsz = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
        const int within = logical - group * width;
        tm = first_m + within % gsz;
        tn = within / gsz;
    }
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- staging assignment: thread -> (row, chunk); addresses = uniform tile base + 32-bit offset ----
    const int lc = tid & 3;       // 16-B chunk within the 64-B k step
    const int lr = tid >> 2;      // row 0..63 (+64 i)
    const char *baseA = g.A + static_cast<int64_t>(m0) * g.Kb;
    const char *baseB = g.Bm + static_cast<int64_t>(n0) * g.Kb;
    uint32_t offa[WM], offb[WN];
    bool oka[WM], okb[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int row = lr + 64 * i;
        oka[i] = m0 + row < g.M;
        offa[i] = static_cast<uint32_t>(oka[i] ? row : 0) * static_cast<uint32_t>(g.Kb) + lc * 16;
    }
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int row = lr + 64 * j;
        okb[j] = n0 + row < g.N;
        offb[j] = static_cast<uint32_t>(okb[j] ? row : 0) * static_cast<uint32_t>(g.Kb) + lc * 16;
    }

    typename Mma<KIND>::acc_t acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::zero();

    u32x4 ra[WM], rb[WN];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int nk = (g.Kb + 63) >> 6;

#define HLQ_LOAD_GLOBAL(KT)                                                                                   \
    {                                                                                                         \
        const uint32_t kofs = static_cast<uint32_t>(KT) * 64u;                                                \
        const bool kok = static_cast<int>(kofs) + lc * 16 < g.Kb;                                             \
        _Pragma("unroll") for (int i = 0; i < WM; ++i)                                                        \
            ra[i] = (oka[i] && kok) ? *reinterpret_cast<const u32x4 *>(baseA + (offa[i] + kofs)) : zero4;     \
        _Pragma("unroll") for (int j = 0; j < WN; ++j)                                                        \
            rb[j] = (okb[j] && kok) ? *reinterpret_cast<const u32x4 *>(baseB + (offb[j] + kofs)) : zero4;     \
    }
#define HLQ_STORE_LDS(STAGE)                                                                                  \
    {                                                                                                         \
        _Pragma("unroll") for (int i = 0; i < WM; ++i) lds[STAGE][lds_chunk(lr + 64 * i, lc)] = ra[i];        \
        _Pragma("unroll") for (int j = 0; j < WN; ++j) lds[STAGE][BM * 4 + lds_chunk(lr + 64 * j, lc)] = rb[j]; \
    }

    HLQ_LOAD_GLOBAL(0)
    HLQ_STORE_LDS(0)
    __syncthreads();

    const int fr = lane & 31;   // row within a 32-row MFMA operand
    const int fh = lane >> 5;   // which 16-B half of the 32-B k slice

    for (int kt = 0; kt < nk; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < nk) HLQ_LOAD_GLOBAL(kt + 1)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            u32x4 fa[WM], fb[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i)
                fa[i] = lds[stage][lds_chunk(wave_m * (32 * WM) + i * 32 + fr, ks * 2 + fh)];
#pragma unroll
            for (int j = 0; j < WN; ++j)
                fb[j] = lds[stage][BM * 4 + lds_chunk(wave_n * (32 * WN) + j * 32 + fr, ks * 2 + fh)];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) acc[i][j] = Mma<KIND>::mma(fb[j], fa[i], acc[i][j]);
        }
        if (kt + 1 < nk) HLQ_STORE_LDS(stage ^ 1)
        __syncthreads();
    }
#undef HLQ_LOAD_GLOBAL
#undef HLQ_STORE_LDS

    // ---- epilogue: lane holds, per accumulator group vg, C[m][n .. n+3] ----
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int m = m0 + wave_m * (32 * WM) + i * 32 + fr;
        if (m >= g.M) continue;
        const float sa = (g.sA ? g.sA[m] : 1.0f);
#pragma unroll
        for (int j = 0; j < WN; ++j) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int n = n0 + wave_n * (32 * WN) + j * 32 + vg * 8 + fh * 4;
                if (n >= g.N) continue;
                const int64_t off = static_cast<int64_t>(m) * g.N + n;
                if (KIND == 0 && g.acc) {
                    int4 raw;
                    raw.x = static_cast<int>(acc[i][j][vg * 4 + 0]);
                    raw.y = static_cast<int>(acc[i][j][vg * 4 + 1]);
                    raw.z = static_cast<int>(acc[i][j][vg * 4 + 2]);
                    raw.w = static_cast<int>(acc[i][j][vg * 4 + 3]);
                    *reinterpret_cast<int4 *>(g.acc + off) = raw;
                }
                if (g.C) {
                    float o[4];
                    if (g.sB) {
                        const float4 sb = *reinterpret_cast<const float4 *>(g.sB + n);
                        o[0] = sb.x; o[1] = sb.y; o[2] = sb.z; o[3] = sb.w;
                    } else {
                        o[0] = o[1] = o[2] = o[3] = 1.0f;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = Mma<KIND>::to_float(acc[i][j][vg * 4 + e]) * (sa * o[e]) * g.alpha;
                    if (g.c_is_f32) {
                        *reinterpret_cast<float4 *>(static_cast<float *>(g.C) + off) = make_float4(o[0], o[1], o[2], o[3]);
                    } else {
                        uint2 p;
                        p.x = pack_bf16(o[0], o[1]);
                        p.y = pack_bf16(o[2], o[3]);
                        *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(g.C) + off) = p;
                    }
                }
            }
        }
    }
}

template <int KIND, int WM, int WN>
static hipError_t launch_t(const GemmArgs &a, hipStream_t st)
{
    GemmDev g;
    g.A = static_cast<const char *>(a.A);
    g.Bm = static_cast<const char *>(a.Bm);
    g.M = a.M;
    g.N = a.N;
    g.Kb = KIND == 0 ? a.K : 2 * a.K;
    g.sA = a.sA;
    g.sB = a.sB;
    g.alpha = a.alpha;
    g.C = a.C;
    g.c_is_f32 = a.c_is_f32 ? 1 : 0;
    g.acc = a.acc;
    g.tiles_m = (a.M + 64 * WM - 1) / (64 * WM);
    g.tiles_n = (a.N + 64 * WN - 1) / (64 * WN);
    hipLaunchKernelGGL((k_gemm_nt<KIND, WM, WN>), dim3(g.tiles_m * g.tiles_n), dim3(256), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_gemm_nt(int kind, const GemmArgs &a, hipStream_t st)
{
    // 256 x 256 tiles when they still give every compute unit work, else 128 x 128
    const int64_t big_tiles = static_cast<int64_t>((a.M + 255) / 256) * ((a.N + 255) / 256);
    const bool big = big_tiles >= 200;
    if (kind == 0) return big ? launch_t<0, 4, 4>(a, st) : launch_t<0, 2, 2>(a, st);
    return big ? launch_t<1, 4, 4>(a, st) : launch_t<1, 2, 2>(a, st);
}

}  // namespace hlq
