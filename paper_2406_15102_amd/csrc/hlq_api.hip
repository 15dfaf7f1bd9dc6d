// C ABI of the library (declared in hlq.h): argument validation, workspace carving, stream-key
// derivation and the launch sequence of the HLQ backward pass (arXiv 2406.15102, Sec. 6.1).
#include "hlq.h"
#include "hlq_kernels.hpp"

#include <mutex>

namespace {

inline size_t up256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }
inline bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Stream key for (seed, tensor): output number tensor+1 of SplitMix64 started at `seed`;
// tensor 0 = the G operand, 1 = the W operand.  Low half keys the counter, high half the mixer.
inline uint64_t stream_key(uint64_t seed, uint32_t tensor)
{
    uint64_t z = seed + (static_cast<uint64_t>(tensor) + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int check_block(int B) { return (B == 16 || B == 32 || B == 64) ? HLQ_OK : HLQ_ERR_BLOCK; }
int check_rank(int B, int r) { return (r >= 1 && r <= B && is_pow2(r)) ? HLQ_OK : HLQ_ERR_RANK; }
int check_dtype(int dt) { return (dt == HLQ_BF16 || dt == HLQ_F32) ? HLQ_OK : HLQ_ERR_DTYPE; }

// rows x K operand of the quantiser: K a multiple of B, K <= 65536 for the row kernel,
// rows*K/4 random words addressable by a 32-bit counter
int check_quant_shape(int64_t rows, int64_t K, int B)
{
    if (rows <= 0 || K <= 0 || K % B != 0 || K > 65536) return HLQ_ERR_SHAPE;
    if (rows > (int64_t(1) << 31) - 1) return HLQ_ERR_SHAPE;
    if (rows * (K / 4) >= (int64_t(1) << 32)) return HLQ_ERR_SHAPE;
    return HLQ_OK;
}

int check_hla_shape(int64_t N, int64_t D, int B, int r)
{
    if (N <= 0 || D <= 0 || N % B != 0 || D % 8 != 0 || D > (int64_t(1) << 30)) return HLQ_ERR_SHAPE;
    const int64_t Kc = N / B * r;
    if (Kc % 8 != 0 || Kc > (int64_t(1) << 30)) return HLQ_ERR_SHAPE;
    if ((N / B + 3) / 4 > 65535) return HLQ_ERR_SHAPE;   // token-block groups are the grid's y axis
    if ((D + 127) / 128 * ((N / B + 3) / 4) >= (int64_t(1) << 30)) return HLQ_ERR_SHAPE;   // workgroups of one launch
    return HLQ_OK;
}

// Longest reduction of the integer products: 127 * 127 * K (8-bit codes) and 256 * 49 * K (packed 4-bit
// codes, accumulated times 256) must stay below 2^31.
constexpr int64_t kMaxIntK = 131072;

int check_gemm_shape(int64_t M, int64_t Nn, int64_t K, int kmult)
{
    if (M <= 0 || Nn <= 0 || K <= 0 || K % kmult != 0 || Nn % 4 != 0) return HLQ_ERR_SHAPE;
    // 32-bit byte offsets inside a 256-row operand tile: 256 rows x (2 K) bytes must stay below 2^31
    if (M > (int64_t(1) << 30) || Nn > (int64_t(1) << 30) || K > (int64_t(1) << 21)) return HLQ_ERR_SHAPE;
    if (((M + 127) / 128) * ((Nn + 127) / 128) > (int64_t(1) << 30)) return HLQ_ERR_SHAPE;
    return HLQ_OK;
}

int check_backward_shape(int64_t N, int64_t d_in, int64_t d_out, int B, int r)
{
    int rc;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_rank(B, r)) != HLQ_OK) return rc;
    if (N <= 0 || d_in <= 0 || d_out <= 0) return HLQ_ERR_SHAPE;
    if (d_in % 8 != 0) return HLQ_ERR_SHAPE;
    if ((rc = check_quant_shape(N, d_out, B)) != HLQ_OK) return rc;
    if ((rc = check_quant_shape(d_in, d_out, B)) != HLQ_OK) return rc;
    if ((rc = check_hla_shape(N, d_in, B, r)) != HLQ_OK) return rc;
    if ((rc = check_hla_shape(N, d_out, B, r)) != HLQ_OK) return rc;
    if ((rc = check_gemm_shape(N, d_in, d_out, 16)) != HLQ_OK) return rc;
    if ((rc = check_gemm_shape(d_out, d_in, N / B * r, 8)) != HLQ_OK) return rc;
    return HLQ_OK;
}

// Carving of the backward workspace.  With HLQ_FLAG_GW_INT8 the compressed operands are int8
// codes with one scale per feature plus one word of column maximum per feature.
struct Layout {
    size_t Gq, sG, Wq, sW, wws, GhatT, sGhat, XhatT, sXhat, hws, gws, gws_bytes, total;
};

Layout make_layout(int64_t N, int64_t d_in, int64_t d_out, int B, int r, bool x_is_compressed, int flags)
{
    Layout L;
    const size_t Kc = static_cast<size_t>(N / B * r);
    const bool gwi = (flags & HLQ_FLAG_GW_INT8) != 0;
    const size_t esz = gwi ? 1 : 2;
    size_t off = 0;
    L.Gq = off;    off += up256(static_cast<size_t>(N) * d_out);
    L.sG = off;    off += up256(static_cast<size_t>(N) * 4);
    L.Wq = off;    off += up256(static_cast<size_t>(d_in) * d_out);
    L.sW = off;    off += up256(static_cast<size_t>(d_in) * 4);
    L.wws = off;   off += up256(hlq::quant_cols_ws_bytes(d_out, d_in));
    // integer g_w list: column maxima of projected G (d_out words), then of projected X (d_in words),
    // right behind those of the weight so that one fill zeroes all three
    L.hws = off;   off += gwi ? up256(hlq::hla_quant_ws_bytes(d_out)) + up256(hlq::hla_quant_ws_bytes(d_in)) : 0;
    L.GhatT = off; off += up256(static_cast<size_t>(d_out) * Kc * esz);
    L.sGhat = off; off += gwi ? up256(static_cast<size_t>(d_out) * 4) : 0;
    // X projected here, or the int8 codes unpacked from a 4-bit store that was handed over
    const bool x_unpack = x_is_compressed && (flags & HLQ_FLAG_XC_INT4);
    L.XhatT = off; off += (x_is_compressed && !x_unpack) ? 0 : up256(static_cast<size_t>(d_in) * Kc * esz);
    L.sXhat = off; off += (gwi && !x_is_compressed) ? up256(static_cast<size_t>(d_in) * 4) : 0;
    // split-K partial sums of whichever product wants them (the two products run one after the other)
    const size_t g1 = hlq::gemm_ws_bytes(0, static_cast<int>(N), static_cast<int>(d_in), static_cast<int>(d_out));
    const size_t g2 = hlq::gemm_ws_bytes(gwi ? 0 : 1, static_cast<int>(d_out), static_cast<int>(d_in), static_cast<int>(Kc));
    L.gws_bytes = g1 > g2 ? g1 : g2;
    if (!(flags & HLQ_FLAG_SEPARATE_PRODUCTS)) {
        // the two products in one launch plan the g_w product's k split for the pair
        const bool packed = !(flags & (HLQ_FLAG_GX_8BIT | HLQ_FLAG_GX_UNPACKED)) && d_out % 32 == 0;
        hlq::GemmArgs ax{}, aw{};
        ax.M = static_cast<int>(N), ax.N = static_cast<int>(d_in), ax.K = static_cast<int>(d_out);
        aw.M = static_cast<int>(d_out), aw.N = static_cast<int>(d_in), aw.K = static_cast<int>(Kc);
        const size_t gp = hlq::gemm_pair_ws_bytes(packed ? 2 : 0, ax, gwi ? 0 : 1, aw, size_t(256) << 20);
        if (gp > L.gws_bytes) L.gws_bytes = gp;
    }
    L.gws = off;   off += up256(L.gws_bytes);
    L.total = off;
    return L;
}

int check_flags(int flags, int r, int64_t N, int B)
{
    if (flags & ~(HLQ_FLAG_GX_8BIT | HLQ_FLAG_GW_INT8 | HLQ_FLAG_GX_UNPACKED | HLQ_FLAG_GW_SEQUENCY | HLQ_FLAG_ROUND_MANTISSA |
                  HLQ_FLAG_SEPARATE_PRODUCTS | HLQ_FLAG_XC_INT4)) return HLQ_ERR_SHAPE;
    if (flags & HLQ_FLAG_GW_INT8) {
        if (r % 4 != 0) return HLQ_ERR_RANK;
        if ((N / B * r) % 16 != 0) return HLQ_ERR_SHAPE;
    }
    if (flags & HLQ_FLAG_XC_INT4) {
        // the 4-bit store belongs to the integer g_w list; its rows are whole 16-byte pieces of packed codes
        if (!(flags & HLQ_FLAG_GW_INT8)) return HLQ_ERR_SHAPE;
        if (r % 8 != 0) return HLQ_ERR_RANK;
        if ((N / B * r) % 32 != 0) return HLQ_ERR_SHAPE;
    }
    return HLQ_OK;
}

inline bool bits_mant(int bits) { return (bits & HLQ_BITS_ROUND_MANTISSA) != 0; }
inline int bits_base(int bits) { return bits & ~HLQ_BITS_ROUND_MANTISSA; }
inline bool bits_ok(int bits)
{
    const int b = bits_base(bits);
    return b == HLQ_BITS_4 || b == HLQ_BITS_8 || b == HLQ_BITS_4_PACKED;
}
inline float bits_qmax(int bits) { return bits_base(bits) == HLQ_BITS_8 ? 127.0f : 7.0f; }
inline bool bits_packed(int bits) { return bits_base(bits) == HLQ_BITS_4_PACKED; }

// Workspace of the calls that pass none: per device, either the memory the caller registered with
// hlq_set_workspace (never allocated, freed or synchronised here), or a library-owned buffer grown on
// demand.
constexpr int kMaxDevices = 64;
std::mutex g_ws_mutex;
void *g_ws_ptr[kMaxDevices] = {nullptr};
size_t g_ws_bytes[kMaxDevices] = {0};
void *g_user_ws_ptr[kMaxDevices] = {nullptr};
size_t g_user_ws_bytes[kMaxDevices] = {0};

// the device the calling thread has current; 0 where no device can be asked (argument checks on a
// machine without a GPU must still come out with their status)
int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return dev;
}

int own_workspace(size_t bytes, void **out)
{
    const int dev = current_device();
    if (dev < 0 || dev >= kMaxDevices) return HLQ_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (g_user_ws_ptr[dev]) {
        // registered by the caller: use it or refuse; nothing is allocated, freed or waited for
        if (g_user_ws_bytes[dev] < bytes) return HLQ_ERR_WORKSPACE;
        *out = g_user_ws_ptr[dev];
        return HLQ_OK;
    }
    if (g_ws_bytes[dev] < bytes) {
        if (g_ws_ptr[dev]) {
            // earlier calls may still be running on the old buffer
            if (hipDeviceSynchronize() != hipSuccess) return HLQ_ERR_WORKSPACE;
            (void)hipFree(g_ws_ptr[dev]);
            g_ws_ptr[dev] = nullptr;
            g_ws_bytes[dev] = 0;
        }
        void *p = nullptr;
        if (hipMalloc(&p, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return HLQ_ERR_WORKSPACE;
        }
        g_ws_ptr[dev] = p;
        g_ws_bytes[dev] = bytes;
    }
    *out = g_ws_ptr[dev];
    return HLQ_OK;
}

inline int launch_rc(hipError_t e) { return e == hipSuccess ? HLQ_OK : HLQ_ERR_LAUNCH; }

}  // namespace

extern "C" {

const char *hlq_status_str(int status)
{
    switch (status) {
        case HLQ_OK: return "HLQ_OK";
        case HLQ_ERR_NULL: return "HLQ_ERR_NULL: a required pointer is NULL";
        case HLQ_ERR_SHAPE: return "HLQ_ERR_SHAPE: a size breaks the shape rules";
        case HLQ_ERR_BLOCK: return "HLQ_ERR_BLOCK: B must be 16, 32 or 64";
        case HLQ_ERR_RANK: return "HLQ_ERR_RANK: r must be a power of two in [1, B]";
        case HLQ_ERR_DTYPE: return "HLQ_ERR_DTYPE: dtype must be HLQ_BF16 or HLQ_F32";
        case HLQ_ERR_WORKSPACE: return "HLQ_ERR_WORKSPACE: workspace too small, misaligned or not allocatable";
        case HLQ_ERR_LAUNCH: return "HLQ_ERR_LAUNCH: the HIP runtime refused a launch";
    }
    return "HLQ: unknown status";
}

int hlq_version(void) { return 200; }

int hlq_set_option(int option, int value)
{
    if (option == HLQ_OPT_PERSISTENT_PRODUCTS) hlq::gemm_stream_enable(value != 0);
    else if (option == HLQ_OPT_SHARED_G_READ) hlq::front_share_enable(value != 0);
    else if (option == HLQ_OPT_DIRECT_TO_LDS) hlq::gemm_dl_enable(value != 0);
    else if (option == HLQ_OPT_TAIL_TILES) hlq::gemm_tail_enable(value != 0);
    else if (option == HLQ_OPT_FRONT_INTERLEAVE) hlq::front_mix_enable(value != 0);
    else if (option == HLQ_OPT_PLAN_TILE && (value == 0 || value == 128 || value == 256)) hlq::gemm_plan_force(value, -1);
    else if (option == HLQ_OPT_PLAN_SPLITS && value >= 0 && value <= 16) hlq::gemm_plan_force(-1, value);
    else return HLQ_ERR_SHAPE;
    return HLQ_OK;
}

int hlq_set_workspace(void *dev_ptr, size_t bytes)
{
    if (dev_ptr && (!aligned(dev_ptr, 256) || bytes == 0)) return HLQ_ERR_WORKSPACE;
    const int dev = current_device();
    if (dev < 0 || dev >= kMaxDevices) return HLQ_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    g_user_ws_ptr[dev] = dev_ptr;
    g_user_ws_bytes[dev] = dev_ptr ? bytes : 0;
    return HLQ_OK;
}

size_t hlq_workspace_bytes(int64_t N, int64_t d_in, int64_t d_out, int B, int r, int x_is_compressed)
{
    if (check_backward_shape(N, d_in, d_out, B, r) != HLQ_OK) return 0;
    return make_layout(N, d_in, d_out, B, r, x_is_compressed != 0, 0).total;
}

size_t hlq_workspace_bytes_mode(int64_t N, int64_t d_in, int64_t d_out, int B, int r, int x_is_compressed, int flags)
{
    if (check_backward_shape(N, d_in, d_out, B, r) != HLQ_OK || check_flags(flags, r, N, B) != HLQ_OK) return 0;
    return make_layout(N, d_in, d_out, B, r, x_is_compressed != 0, flags).total;
}

int hlq_quantize_g(const void *G, int64_t N, int64_t d_out, int B, uint64_t seed, int dtype, int bits, int8_t *Gq,
                   float *sG, float *coeff, void *stream)
{
    int rc;
    if (!G || !Gq || !sG) return HLQ_ERR_NULL;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if (!bits_ok(bits)) return HLQ_ERR_DTYPE;
    if ((rc = check_quant_shape(N, d_out, B)) != HLQ_OK) return rc;
    if (bits_packed(bits) && d_out % 32 != 0) return HLQ_ERR_SHAPE;   // 16-byte rows of packed codes
    if (!aligned(G, 16) || !aligned(Gq, 8) || (coeff && !aligned(coeff, 16))) return HLQ_ERR_SHAPE;
    const uint64_t key = stream_key(seed, 0);
    return launch_rc(hlq::launch_quant_rows(G, N, static_cast<int>(d_out), B, dtype == HLQ_F32,
                                            static_cast<uint32_t>(key), static_cast<uint32_t>(key >> 32),
                                            bits_qmax(bits), bits_packed(bits), bits_mant(bits), Gq, sG, coeff,
                                            static_cast<hipStream_t>(stream)));
}

size_t hlq_quantize_w_workspace_bytes(int64_t d_out, int64_t d_in)
{
    if (d_out <= 0 || d_in <= 0) return 0;
    return hlq::quant_cols_ws_bytes(d_out, d_in);
}

int hlq_quantize_w(const void *W, int64_t d_out, int64_t d_in, int B, uint64_t seed, int dtype, int bits, int8_t *WqT,
                   float *sW, float *coeffT, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc;
    if (!W || !WqT || !sW || !workspace) return HLQ_ERR_NULL;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if (!bits_ok(bits)) return HLQ_ERR_DTYPE;
    if (d_in <= 0 || d_in % 8 != 0) return HLQ_ERR_SHAPE;
    if ((rc = check_quant_shape(d_in, d_out, B)) != HLQ_OK) return rc;
    if (bits_packed(bits) && d_out % 32 != 0) return HLQ_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(WqT, 16) || (coeffT && !aligned(coeffT, 16))) return HLQ_ERR_SHAPE;
    if (!aligned(workspace, 256) || workspace_bytes < hlq::quant_cols_ws_bytes(d_out, d_in)) return HLQ_ERR_WORKSPACE;
    const uint64_t key = stream_key(seed, 1);
    return launch_rc(hlq::launch_quant_cols(W, static_cast<int>(d_out), static_cast<int>(d_in), B, dtype == HLQ_F32,
                                            static_cast<uint32_t>(key), static_cast<uint32_t>(key >> 32),
                                            bits_qmax(bits), bits_packed(bits), bits_mant(bits), WqT, sW, coeffT, workspace,
                                            static_cast<hipStream_t>(stream)));
}

int hlq_quantize_w_static(const void *W, int64_t d_out, int64_t d_in, int B, uint64_t seed, int dtype, int bits,
                          int8_t *WqT, float *sW, void *stream)
{
    int rc;
    if (!W || !WqT || !sW) return HLQ_ERR_NULL;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if (!bits_ok(bits)) return HLQ_ERR_DTYPE;
    if (d_in <= 0 || d_in % 8 != 0) return HLQ_ERR_SHAPE;
    if ((rc = check_quant_shape(d_in, d_out, B)) != HLQ_OK) return rc;
    if (bits_packed(bits) && d_out % 32 != 0) return HLQ_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(WqT, 16)) return HLQ_ERR_SHAPE;
    if (d_in > hlq::kQuantColsStaticMaxI) return HLQ_ERR_WORKSPACE;   // beyond the library's static scratch
    void *ws = nullptr;
    if (hlq::quant_cols_static_scratch(&ws) != hipSuccess) {
        (void)hipGetLastError();
        return HLQ_ERR_WORKSPACE;
    }
    const uint64_t key = stream_key(seed, 1);
    return launch_rc(hlq::launch_quant_cols(W, static_cast<int>(d_out), static_cast<int>(d_in), B, dtype == HLQ_F32,
                                            static_cast<uint32_t>(key), static_cast<uint32_t>(key >> 32),
                                            bits_qmax(bits), bits_packed(bits), bits_mant(bits), WqT, sW, nullptr, ws,
                                            static_cast<hipStream_t>(stream)));
}

size_t hlq_gemm_workspace_bytes(int kind, int64_t M, int64_t Nn, int64_t K)
{
    if (kind < 0 || kind > 2 || check_gemm_shape(M, Nn, K, kind == 0 ? 16 : (kind == 1 ? 8 : 32)) != HLQ_OK) return 0;
    if (kind != 1 && K > kMaxIntK) return 0;
    return hlq::gemm_ws_bytes(kind, static_cast<int>(M), static_cast<int>(Nn), static_cast<int>(K));
}

int hlq_int8_gemm_nt(const int8_t *A, const int8_t *Bm, int64_t M, int64_t Nn, int64_t K, const float *sA,
                     const float *sB, float alpha, int out_dtype, void *C, int32_t *acc, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    int rc;
    if (!A || !Bm || (!C && !acc)) return HLQ_ERR_NULL;
    if ((rc = check_dtype(out_dtype)) != HLQ_OK) return rc;
    if ((rc = check_gemm_shape(M, Nn, K, 16)) != HLQ_OK) return rc;
    if (K > kMaxIntK) return HLQ_ERR_SHAPE;
    if (!aligned(A, 16) || !aligned(Bm, 16) || (C && !aligned(C, 16)) || (acc && !aligned(acc, 16)) ||
        (sB && !aligned(sB, 16)))
        return HLQ_ERR_SHAPE;
    if (workspace && !aligned(workspace, 16)) return HLQ_ERR_WORKSPACE;
    hlq::GemmArgs a{A, Bm, static_cast<int>(M), static_cast<int>(Nn), static_cast<int>(K), sA, sB, alpha, C,
                    out_dtype == HLQ_F32, acc, workspace, workspace_bytes};
    return launch_rc(hlq::launch_gemm_nt(0, a, static_cast<hipStream_t>(stream)));
}

int hlq_int4_gemm_nt(const void *A, const void *Bm, int64_t M, int64_t Nn, int64_t K, const float *sA,
                     const float *sB, float alpha, int out_dtype, void *C, int32_t *acc, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    int rc;
    if (!A || !Bm || (!C && !acc)) return HLQ_ERR_NULL;
    if ((rc = check_dtype(out_dtype)) != HLQ_OK) return rc;
    if ((rc = check_gemm_shape(M, Nn, K, 32)) != HLQ_OK) return rc;
    if (K > kMaxIntK) return HLQ_ERR_SHAPE;   // 256 * 49 * K must fit the int32 accumulators
    if (!aligned(A, 16) || !aligned(Bm, 16) || (C && !aligned(C, 16)) || (acc && !aligned(acc, 16)) ||
        (sB && !aligned(sB, 16)))
        return HLQ_ERR_SHAPE;
    if (workspace && !aligned(workspace, 16)) return HLQ_ERR_WORKSPACE;
    hlq::GemmArgs a{A, Bm, static_cast<int>(M), static_cast<int>(Nn), static_cast<int>(K), sA, sB, alpha, C,
                    out_dtype == HLQ_F32, acc, workspace, workspace_bytes};
    return launch_rc(hlq::launch_gemm_nt(2, a, static_cast<hipStream_t>(stream)));
}

// kinds of the two products from the storage of their operands
static int products_kinds(int gx_bits, bool gw_int8, int *kx, int *kw)
{
    if (gx_bits != HLQ_BITS_4 && gx_bits != HLQ_BITS_8 && gx_bits != HLQ_BITS_4_PACKED) return HLQ_ERR_SHAPE;
    *kx = gx_bits == HLQ_BITS_4_PACKED ? 2 : 0;
    *kw = gw_int8 ? 0 : 1;
    return HLQ_OK;
}

static int products_check(int64_t N, int64_t d_in, int64_t d_out, int64_t Kc, int kx, int kw)
{
    int rc;
    if ((rc = check_gemm_shape(N, d_in, d_out, kx == 2 ? 32 : 16)) != HLQ_OK) return rc;
    if ((rc = check_gemm_shape(d_out, d_in, Kc, kw == 0 ? 16 : 8)) != HLQ_OK) return rc;
    if (d_out > kMaxIntK || (kw == 0 && Kc > kMaxIntK)) return HLQ_ERR_SHAPE;
    return HLQ_OK;
}

size_t hlq_backward_products_workspace_bytes(int64_t N, int64_t d_in, int64_t d_out, int64_t Kc, int gx_bits, int gw_int8)
{
    int kx, kw;
    if (products_kinds(gx_bits, gw_int8 != 0, &kx, &kw) != HLQ_OK || products_check(N, d_in, d_out, Kc, kx, kw) != HLQ_OK)
        return 0;
    hlq::GemmArgs ax{}, aw{};
    ax.M = static_cast<int>(N), ax.N = static_cast<int>(d_in), ax.K = static_cast<int>(d_out);
    aw.M = static_cast<int>(d_out), aw.N = static_cast<int>(d_in), aw.K = static_cast<int>(Kc);
    return hlq::gemm_pair_ws_bytes(kx, ax, kw, aw, size_t(256) << 20);
}

int hlq_backward_products_plan(int64_t N, int64_t d_in, int64_t d_out, int64_t Kc, int gx_bits, int gw_int8,
                               size_t workspace_bytes, int *plan)
{
    int rc, kx, kw;
    if (!plan) return HLQ_ERR_NULL;
    if ((rc = products_kinds(gx_bits, gw_int8 != 0, &kx, &kw)) != HLQ_OK) return rc;
    if ((rc = products_check(N, d_in, d_out, Kc, kx, kw)) != HLQ_OK) return rc;
    hlq::GemmArgs ax{}, aw{};
    ax.M = static_cast<int>(N), ax.N = static_cast<int>(d_in), ax.K = static_cast<int>(d_out);
    aw.M = static_cast<int>(d_out), aw.N = static_cast<int>(d_in), aw.K = static_cast<int>(Kc);
    // non-null outputs: the persistent form is only chosen for products that write C
    ax.C = aw.C = plan;
    hlq::gemm_pair_describe(kx, ax, kw, aw, workspace_bytes, plan);
    return HLQ_OK;
}

int hlq_backward_products(const void *Gq, const float *sG, const void *WqT, const float *sW, int gx_bits,
                          const void *GhatT, const float *sGhat, const void *XhatT, const float *sXhat, int64_t N,
                          int64_t d_in, int64_t d_out, int64_t Kc, int B, int dtype, void *dX, void *dW, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    int rc, kx, kw;
    if (!Gq || !sG || !WqT || !sW || !GhatT || !XhatT || !dX || !dW) return HLQ_ERR_NULL;
    if ((sGhat == nullptr) != (sXhat == nullptr)) return HLQ_ERR_NULL;      // both int8 with scales, or both bf16
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if ((rc = products_kinds(gx_bits, sGhat != nullptr, &kx, &kw)) != HLQ_OK) return rc;
    if ((rc = products_check(N, d_in, d_out, Kc, kx, kw)) != HLQ_OK) return rc;
    if (!aligned(Gq, 16) || !aligned(WqT, 16) || !aligned(sW, 16) || !aligned(GhatT, 16) || !aligned(XhatT, 16) ||
        (sXhat && !aligned(sXhat, 16)) || !aligned(dX, 16) || !aligned(dW, 16))
        return HLQ_ERR_SHAPE;
    if (workspace && !aligned(workspace, 16)) return HLQ_ERR_WORKSPACE;
    const float invB = 1.0f / static_cast<float>(B);
    const bool f32 = dtype == HLQ_F32;
    hlq::GemmArgs ax{Gq, WqT, static_cast<int>(N), static_cast<int>(d_in), static_cast<int>(d_out), sG, sW, invB, dX, f32,
                     nullptr, nullptr, 0};
    hlq::GemmArgs aw{GhatT, XhatT, static_cast<int>(d_out), static_cast<int>(d_in), static_cast<int>(Kc), sGhat, sXhat,
                     invB, dW, f32, nullptr, workspace, workspace_bytes};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hlq::gemm_pair_available(kx, ax, kw, aw)) return launch_rc(hlq::launch_gemm_pair(kx, ax, kw, aw, st));
    // a grid too large for one launch: one launch per product
    if ((rc = launch_rc(hlq::launch_gemm_nt(kx, ax, st))) != HLQ_OK) return rc;
    return launch_rc(hlq::launch_gemm_nt(kw, aw, st));
}

int hlq_hla_project(const void *T, int64_t N, int64_t D, int B, int r, int dtype, void *ThatT, float *coeffT,
                    void *stream)
{
    return hlq_hla_project_basis(T, N, D, B, r, HLQ_BASIS_NATURAL, dtype, ThatT, coeffT, stream);
}

int hlq_hla_project_basis(const void *T, int64_t N, int64_t D, int B, int r, int basis, int dtype, void *ThatT,
                          float *coeffT, void *stream)
{
    int rc;
    if (!T || !ThatT) return HLQ_ERR_NULL;
    if (basis != HLQ_BASIS_NATURAL && basis != HLQ_BASIS_SEQUENCY) return HLQ_ERR_RANK;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_rank(B, r)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if ((rc = check_hla_shape(N, D, B, r)) != HLQ_OK) return rc;
    if (!aligned(T, 16) || !aligned(ThatT, 16) || (coeffT && !aligned(coeffT, 16))) return HLQ_ERR_SHAPE;
    return launch_rc(hlq::launch_hla(T, N, static_cast<int>(D), B, r, basis, dtype == HLQ_F32,
                                     static_cast<uint16_t *>(ThatT), coeffT, static_cast<hipStream_t>(stream)));
}

int hlq_compress_act(const void *X, int64_t N, int64_t d_in, int B, int r, int dtype, void *XhatT, void *stream)
{
    return hlq_hla_project(X, N, d_in, B, r, dtype, XhatT, nullptr, stream);
}

int hlq_bf16_gemm_nt(const void *A, const void *Bm, int64_t M, int64_t Nn, int64_t K, float alpha, int out_dtype,
                     void *C, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc;
    if (!A || !Bm || !C) return HLQ_ERR_NULL;
    if ((rc = check_dtype(out_dtype)) != HLQ_OK) return rc;
    if ((rc = check_gemm_shape(M, Nn, K, 8)) != HLQ_OK) return rc;
    if (!aligned(A, 16) || !aligned(Bm, 16) || !aligned(C, 16)) return HLQ_ERR_SHAPE;
    if (workspace && !aligned(workspace, 16)) return HLQ_ERR_WORKSPACE;
    hlq::GemmArgs a{A, Bm, static_cast<int>(M), static_cast<int>(Nn), static_cast<int>(K), nullptr, nullptr, alpha, C,
                    out_dtype == HLQ_F32, nullptr, workspace, workspace_bytes};
    return launch_rc(hlq::launch_gemm_nt(1, a, static_cast<hipStream_t>(stream)));
}

int hlq_mfma_probe(int kind, int blocks, int iters, float *sink, void *stream)
{
    if (!sink) return HLQ_ERR_NULL;
    if (kind < 0 || kind > 9 || blocks <= 0 || blocks > (1 << 20) || iters <= 0) return HLQ_ERR_SHAPE;
    return launch_rc(hlq::launch_mfma_probe(kind, blocks, iters, sink, static_cast<hipStream_t>(stream)));
}

size_t hlq_hla_quantize_workspace_bytes(int64_t D) { return D > 0 ? hlq::hla_quant_ws_bytes(D) : 0; }

int hlq_hla_quantize(const void *T, int64_t N, int64_t D, int B, int r, uint64_t seed, int tensor, int dtype,
                     int8_t *TqT, float *sT, float *coeffT, void *workspace, size_t workspace_bytes, void *stream)
{
    return hlq_hla_quantize_basis(T, N, D, B, r, HLQ_BASIS_NATURAL, seed, tensor, dtype, TqT, sT, coeffT, workspace,
                                  workspace_bytes, stream);
}

int hlq_hla_quantize_basis(const void *T, int64_t N, int64_t D, int B, int r, int basis, uint64_t seed, int tensor,
                           int dtype, int8_t *TqT, float *sT, float *coeffT, void *workspace, size_t workspace_bytes,
                           void *stream)
{
    int rc;
    if (!T || !TqT || !sT || !workspace) return HLQ_ERR_NULL;
    const bool mant = (basis & HLQ_BASIS_ROUND_MANTISSA) != 0;
    basis &= ~HLQ_BASIS_ROUND_MANTISSA;
    if (basis != HLQ_BASIS_NATURAL && basis != HLQ_BASIS_SEQUENCY) return HLQ_ERR_RANK;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_rank(B, r)) != HLQ_OK) return rc;
    if (r % 4 != 0) return HLQ_ERR_RANK;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if ((rc = check_hla_shape(N, D, B, r)) != HLQ_OK) return rc;
    if (tensor != 2 && tensor != 3) return HLQ_ERR_SHAPE;
    const int64_t Kc = N / B * r;
    if (Kc % 16 != 0 || D * (Kc / 4) >= (int64_t(1) << 32)) return HLQ_ERR_SHAPE;
    if (!aligned(T, 16) || !aligned(TqT, 16) || (coeffT && !aligned(coeffT, 16))) return HLQ_ERR_SHAPE;
    if (!aligned(workspace, 256) || workspace_bytes < hlq::hla_quant_ws_bytes(D)) return HLQ_ERR_WORKSPACE;
    const uint64_t key = stream_key(seed, static_cast<uint32_t>(tensor));
    return launch_rc(hlq::launch_hla_quant(T, N, static_cast<int>(D), B, r, basis, dtype == HLQ_F32,
                                           static_cast<uint32_t>(key), static_cast<uint32_t>(key >> 32), mant, TqT, sT,
                                           coeffT, workspace, static_cast<hipStream_t>(stream)));
}

int hlq_compress_act_int8(const void *X, int64_t N, int64_t d_in, int B, int r, uint64_t seed, int dtype,
                          int8_t *XqT, float *sX, void *workspace, size_t workspace_bytes, void *stream)
{
    return hlq_hla_quantize(X, N, d_in, B, r, seed, 2, dtype, XqT, sX, nullptr, workspace, workspace_bytes, stream);
}

int hlq_compress_act_int4(const void *X, int64_t N, int64_t d_in, int B, int r, uint64_t seed, int dtype, uint8_t *Xq4T,
                          float *sX, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc;
    if (!X || !Xq4T || !sX || !workspace) return HLQ_ERR_NULL;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_rank(B, r)) != HLQ_OK) return rc;
    if (r % 8 != 0) return HLQ_ERR_RANK;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if ((rc = check_hla_shape(N, d_in, B, r)) != HLQ_OK) return rc;
    const int64_t Kc = N / B * r;
    if (Kc % 32 != 0 || d_in * (Kc / 4) >= (int64_t(1) << 32)) return HLQ_ERR_SHAPE;
    if (!aligned(X, 16) || !aligned(Xq4T, 16)) return HLQ_ERR_SHAPE;
    if (!aligned(workspace, 256) || workspace_bytes < hlq::hla_quant_ws_bytes(d_in)) return HLQ_ERR_WORKSPACE;
    const uint64_t key = stream_key(seed, 2);
    return launch_rc(hlq::launch_hla_quant(X, N, static_cast<int>(d_in), B, r, HLQ_BASIS_NATURAL, dtype == HLQ_F32,
                                           static_cast<uint32_t>(key), static_cast<uint32_t>(key >> 32), false,
                                           reinterpret_cast<int8_t *>(Xq4T), sX, nullptr, workspace,
                                           static_cast<hipStream_t>(stream), true));
}

// The whole path.  Either W (quantised here, every call) or its codes and scales as hlq_quantize_w
// left them (Wc, sWc): the weight changes once per optimiser step, not once per micro-batch.
// Everything backward_impl refuses, tested before the first launch.
static int backward_check(const void *G, const void *X, const void *Xc, const float *sXc, const void *W, const void *Wc,
                          const float *sWc, int64_t N, int64_t d_in, int64_t d_out, int B, int r, int dtype, int flags,
                          const void *dX, const void *dW)
{
    int rc;
    if ((rc = check_backward_shape(N, d_in, d_out, B, r)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if ((rc = check_flags(flags, r, N, B)) != HLQ_OK) return rc;
    const bool gwi = (flags & HLQ_FLAG_GW_INT8) != 0;
    if (!G || (!dX && !dW)) return HLQ_ERR_NULL;
    if (dX && !W && !(Wc && sWc)) return HLQ_ERR_NULL;
    if (Wc && (!aligned(Wc, 16) || !aligned(sWc, 16))) return HLQ_ERR_SHAPE;
    if (dW && ((X == nullptr) == (Xc == nullptr))) return HLQ_ERR_NULL;   // exactly one of the two
    if (dW && Xc && (gwi != (sXc != nullptr))) return HLQ_ERR_NULL;       // int8 codes come with their scales
    if ((flags & HLQ_FLAG_XC_INT4) && dW && !Xc) return HLQ_ERR_NULL;     // the flag describes a store that is handed over
    if (!aligned(G, 16) || (X && !aligned(X, 16)) || (Xc && !aligned(Xc, 16)) || (sXc && !aligned(sXc, 16)) ||
        (W && !aligned(W, 16)) || (dX && !aligned(dX, 16)) || (dW && !aligned(dW, 16)))
        return HLQ_ERR_SHAPE;
    if (gwi && static_cast<int64_t>(d_out > d_in ? d_out : d_in) * (N / B * r / 4) >= (int64_t(1) << 32))
        return HLQ_ERR_SHAPE;
    if (gwi && N / B * r > kMaxIntK) return HLQ_ERR_SHAPE;   // int32 accumulators of the int8 dW product
    return HLQ_OK;
}

// conv: NULL, or the geometry of a convolution; X is then its channels-last image and stands for
// the column matrix [N, d_in], which the g_w list reads through the image (hla_conv_ok required).
static int backward_impl(const void *G, const void *X, const void *Xc, const float *sXc, const void *W, const void *Wc,
                         const float *sWc, int64_t N, int64_t d_in, int64_t d_out, int B, int r, uint64_t seed, int dtype,
                         int flags, void *dX, void *dW, void *workspace, size_t workspace_bytes, void *stream,
                         const hlq::ConvShape *conv = nullptr, hlq::SplitReduce *defer = nullptr)
{
    if (defer) defer->blocks = 0;
    int rc;
    if ((rc = backward_check(G, X, Xc, sXc, W, Wc, sWc, N, d_in, d_out, B, r, dtype, flags, dX, dW)) != HLQ_OK) return rc;
    const bool gwi = (flags & HLQ_FLAG_GW_INT8) != 0;
    const float qmax = (flags & HLQ_FLAG_GX_8BIT) ? 127.0f : 7.0f;
    // 4-bit codes travel two to a byte whenever their rows stay 16-byte aligned that way
    const bool packed = !(flags & (HLQ_FLAG_GX_8BIT | HLQ_FLAG_GX_UNPACKED)) && d_out % 32 == 0;
    const int basis = (flags & HLQ_FLAG_GW_SEQUENCY) ? HLQ_BASIS_SEQUENCY : HLQ_BASIS_NATURAL;
    const bool mant = (flags & HLQ_FLAG_ROUND_MANTISSA) != 0;

    const bool xc = (Xc != nullptr) || !dW;   // no projection of X is held here: it was handed over, or dW is not wanted
    const Layout L = make_layout(N, d_in, d_out, B, r, xc, flags);
    char *ws = static_cast<char *>(workspace);
    if (ws) {
        if (!aligned(ws, 256) || workspace_bytes < L.total) return HLQ_ERR_WORKSPACE;
    } else {
        void *p = nullptr;
        if ((rc = own_workspace(L.total, &p)) != HLQ_OK) return rc;
        ws = static_cast<char *>(p);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool f32 = dtype == HLQ_F32;
    const int O = static_cast<int>(d_out), I = static_cast<int>(d_in);
    const int Kc = static_cast<int>(N / B * r);
    const float invB = 1.0f / static_cast<float>(B);

    // Launch order: the readers of G next to each other (the second one finds it in the last-level
    // cache), the two passes over W back to back, then the two products.
    int8_t *Gq = reinterpret_cast<int8_t *>(ws + L.Gq);
    float *sG = reinterpret_cast<float *>(ws + L.sG);
    const bool wc = (Wc != nullptr);
    const int8_t *Wq = wc ? static_cast<const int8_t *>(Wc) : reinterpret_cast<const int8_t *>(ws + L.Wq);
    const float *sW = wc ? sWc : reinterpret_cast<const float *>(ws + L.sW);
    void *Gh = ws + L.GhatT;
    float *sGh = reinterpret_cast<float *>(ws + L.sGhat);
    const void *Xh = Xc;
    const float *sXh = sXc;
    if (dW && Xc && (flags & HLQ_FLAG_XC_INT4)) {
        // the activation was kept as 4-bit codes (Sec. 6.1): widen them to the int8 operand of the product
        int8_t *xu = reinterpret_cast<int8_t *>(ws + L.XhatT);
        if ((rc = launch_rc(hlq::launch_unpack_nibbles(Xc, xu, static_cast<int64_t>(d_in) * Kc / 2, st))) != HLQ_OK) return rc;
        Xh = xu;
    }
    // The transforms that depend on nothing share launches when the shapes allow (k_front.hip): two
    // and pass 2 over the weight for the default path (one in all when the weight has few rows or
    // is not transformed here), three for the integer g_w list.  Very long rows of G and the mantissa-bit rounding keep one
    // launch per stage.
    const bool fusable = hlq::front_fusable(O, B) && !mant;   // the fused launches carry the seeded rounding only
    const bool fused = !gwi && fusable;
    const bool fused_q = gwi && fusable;
    const uint64_t kg = stream_key(seed, 0);
    if (fused_q) {
        uint32_t *amax_w = reinterpret_cast<uint32_t *>(ws + L.wws);
        uint32_t *amax_g = reinterpret_cast<uint32_t *>(ws + L.hws);
        uint32_t *amax_x = reinterpret_cast<uint32_t *>(ws + L.hws + up256(hlq::hla_quant_ws_bytes(O)));
        const size_t zero_bytes = (L.hws - L.wws) + up256(hlq::hla_quant_ws_bytes(O)) + up256(hlq::hla_quant_ws_bytes(I));
        const uint64_t k3 = stream_key(seed, 3), k2 = stream_key(seed, 2), kw = stream_key(seed, 1);
        const hlq::FrontRows jr = hlq::front_rows(dX ? G : nullptr, N, O, B, static_cast<uint32_t>(kg),
                                                  static_cast<uint32_t>(kg >> 32), qmax, Gq, sG);
        const hlq::FrontFill jf{amax_w, static_cast<int>(zero_bytes / 4)};
        const hlq::FrontHla none = hlq::front_hla(nullptr, N, O, B, r, nullptr);
        const hlq::FrontAbsmax none_w = hlq::front_absmax(nullptr, O, I, B, nullptr);
        // the zeroing first; the row quantiser with it, or -- in turns -- beside the three passes that only read
        const bool k1_later = hlq::front_mix_enabled();
        const hlq::FrontRows no_rows = hlq::front_rows(nullptr, N, O, B, 0, 0, qmax, nullptr, nullptr);
        if ((rc = launch_rc(hlq::launch_front(k1_later ? no_rows : jr, none, jf, none, none_w, nullptr, B, basis, f32, packed, st))) != HLQ_OK)
            return rc;
        int8_t *xq = xc ? nullptr : reinterpret_cast<int8_t *>(ws + L.XhatT);
        float *sx = xc ? nullptr : reinterpret_cast<float *>(ws + L.sXhat);
        if (conv && dW && !xc) {
            // the image's projection keeps its own launches (it zeroes its maxima itself)
            if ((rc = launch_rc(hlq::launch_hla_quant_conv(X, *conv, B, r, basis, f32, static_cast<uint32_t>(k2),
                                                           static_cast<uint32_t>(k2 >> 32), mant, xq, sx, nullptr, amax_x,
                                                           st))) != HLQ_OK)
                return rc;
        }
        const hlq::FrontHlaQ jg = hlq::front_hlaq(dW ? G : nullptr, N, O, B, r, amax_g, static_cast<uint32_t>(k3),
                                                  static_cast<uint32_t>(k3 >> 32), static_cast<int8_t *>(Gh), sGh);
        const hlq::FrontHlaQ jx = hlq::front_hlaq(dW && !xc && !conv ? X : nullptr, N, I, B, r, amax_x, static_cast<uint32_t>(k2),
                                                  static_cast<uint32_t>(k2 >> 32), xq, sx);
        const bool wq = dX && !wc;
        const hlq::FrontAbsmax jw = hlq::front_absmax(wq ? W : nullptr, O, I, B, amax_w);
        const hlq::FrontColsQ jq = hlq::front_colsq(wq ? W : nullptr, O, I, B, amax_w, static_cast<uint32_t>(kw),
                                                    static_cast<uint32_t>(kw >> 32), qmax, reinterpret_cast<int8_t *>(ws + L.Wq),
                                                    reinterpret_cast<float *>(ws + L.sW));
        if ((rc = launch_rc(hlq::launch_front_q(jg, jx, jw, jq, k1_later ? jr : no_rows, B, basis, f32, packed, st))) != HLQ_OK) return rc;
        if (dW && !xc) {
            Xh = xq;
            sXh = sx;
        }
    }
    // g_x stages 3-4, Q(H^T W) transposed: where the codes go, and whether the front launch made them
    const uint64_t kw = stream_key(seed, 1);
    int8_t *const wq = reinterpret_cast<int8_t *>(ws + L.Wq);
    float *const sw = reinterpret_cast<float *>(ws + L.sW);
    bool w_done = wc || fused_q || !dX;   // handed over by the caller, made by the fused launches above, or not needed
    if (fused) {
        uint16_t *xh = xc ? nullptr : reinterpret_cast<uint16_t *>(ws + L.XhatT);
        const hlq::FrontRows jr = hlq::front_rows(dX ? G : nullptr, N, O, B, static_cast<uint32_t>(kg),
                                                  static_cast<uint32_t>(kg >> 32), qmax, Gq, sG);
        const hlq::FrontHla jx = hlq::front_hla(dW && !xc ? X : nullptr, N, I, B, r, xh);
        const hlq::FrontHla jg = hlq::front_hla(dW ? G : nullptr, N, O, B, r, static_cast<uint16_t *>(Gh));
        if (w_done && !conv && hlq::front_mix_enabled()) {
            // no pass over W here: the front launch alone (its second launch has nothing to do), with the
            // quantiser's and the projections' workgroups in turns
            const hlq::FrontAbsmax none_w = hlq::front_absmax(nullptr, O, I, B, nullptr);
            const hlq::FrontFill no_fill{nullptr, 0};
            rc = launch_rc(hlq::launch_front(jr, jg, no_fill, jx, none_w, nullptr, B, basis, f32, packed, st));
        } else if (w_done || hlq::cols_full_ok(O, I, B, f32)) {
            // no pass over W here (a convolution, or the turns switched off), or a weight of few rows, which one
            // workgroup per strip of columns quantises completely: everything independent in one launch
            const hlq::FrontColsQ jq = hlq::front_cols_full(w_done ? nullptr : W, O, I, B, static_cast<uint32_t>(kw),
                                                            static_cast<uint32_t>(kw >> 32), qmax, wq, sw);
            rc = launch_rc(hlq::launch_front_one(jr, jx, jg, jq, conv, B, basis, f32, packed, st));
            w_done = true;
        } else {
            // pass 1 over W rides in the second launch, behind the zeroing of its maxima in the first
            const hlq::FrontAbsmax jw = hlq::front_absmax(W, O, I, B, reinterpret_cast<uint32_t *>(ws + L.wws));
            const hlq::FrontFill jf{reinterpret_cast<uint32_t *>(ws + L.wws), I};
            // The first launch takes K1(G) and K3(G) -- and, unless HLQ_OPT_FRONT_INTERLEAVE is off, K3(X) too,
            // see launch_front_t --, the second what is left and pass 1.  The projection straight from an
            // image exists for the first launch only, so a convolution has K3(X) there and K3(G) in the second.
            if (conv) rc = launch_rc(hlq::launch_front(jr, jx, jf, jg, jw, conv, B, basis, f32, packed, st));
            else rc = launch_rc(hlq::launch_front(jr, jg, jf, jx, jw, nullptr, B, basis, f32, packed, st));
        }
        if (rc != HLQ_OK) return rc;
        if (dW && !xc) Xh = xh;
    }
    if (dX && !fused && !fused_q) {
        // g_x stages 1-2: Q(G H)
        if ((rc = launch_rc(hlq::launch_quant_rows(G, N, O, B, f32, static_cast<uint32_t>(kg),
                                                   static_cast<uint32_t>(kg >> 32), qmax, packed, mant, Gq, sG, nullptr, st))) != HLQ_OK)
            return rc;
    }
    if (dW && !gwi && !fused) {
        // g_w stages 3 and 1 kept in bf16: HLA of G and (unless it was compressed at forward time) of X
        if ((rc = launch_rc(hlq::launch_hla(G, N, O, B, r, basis, f32, static_cast<uint16_t *>(Gh), nullptr, st))) != HLQ_OK) return rc;
        if (!xc) {
            uint16_t *xh = reinterpret_cast<uint16_t *>(ws + L.XhatT);
            rc = launch_rc(conv ? hlq::launch_hla_conv(X, *conv, B, r, basis, f32, xh, nullptr, st)
                                : hlq::launch_hla(X, N, I, B, r, basis, f32, xh, nullptr, st));
            if (rc != HLQ_OK) return rc;
            Xh = xh;
        }
    }
    if (dW && gwi && !fused_q) {
        // g_w stages 3-4 and 1-2: HLA + int8 quantisation of G (stream 3) and of X (stream 2)
        const uint64_t k3 = stream_key(seed, 3), k2 = stream_key(seed, 2);
        if ((rc = launch_rc(hlq::launch_hla_quant(G, N, O, B, r, basis, f32, static_cast<uint32_t>(k3),
                                                  static_cast<uint32_t>(k3 >> 32), mant, static_cast<int8_t *>(Gh), sGh,
                                                  nullptr, ws + L.hws, st))) != HLQ_OK)
            return rc;
        if (!xc) {
            int8_t *xq = reinterpret_cast<int8_t *>(ws + L.XhatT);
            float *sx = reinterpret_cast<float *>(ws + L.sXhat);
            rc = launch_rc(conv ? hlq::launch_hla_quant_conv(X, *conv, B, r, basis, f32, static_cast<uint32_t>(k2),
                                                             static_cast<uint32_t>(k2 >> 32), mant, xq, sx, nullptr,
                                                             ws + L.hws, st)
                                : hlq::launch_hla_quant(X, N, I, B, r, basis, f32, static_cast<uint32_t>(k2),
                                                        static_cast<uint32_t>(k2 >> 32), mant, xq, sx, nullptr, ws + L.hws,
                                                        st));
            if (rc != HLQ_OK) return rc;
            Xh = xq;
            sXh = sx;
        }
    }
    if (!w_done) {
        if (fused)   // pass 1 ran in the second front launch
            rc = launch_rc(hlq::launch_quant_cols_pass2(W, O, I, B, f32, static_cast<uint32_t>(kw),
                                                        static_cast<uint32_t>(kw >> 32), qmax, packed, false, wq, sw,
                                                        nullptr, ws + L.wws, st));
        else
            rc = launch_rc(hlq::launch_quant_cols(W, O, I, B, f32, static_cast<uint32_t>(kw),
                                                  static_cast<uint32_t>(kw >> 32), qmax, packed, mant, wq, sw, nullptr,
                                                  ws + L.wws, st));
        if (rc != HLQ_OK) return rc;
    }
    // The products: g_x stages 5-6 (integer product and dequantisation; 1/B undoes H H^T = B I) and
    // g_w stage 5 (and 6) over the compressed token axis.  Independent of each other: one launch
    // carries both when that combination of kernels is built (k_gemm_pair.hip).
    hlq::GemmArgs ax{Gq, Wq, static_cast<int>(N), I, O, sG, sW, invB, dX, f32, nullptr, ws + L.gws, L.gws_bytes};
    hlq::GemmArgs aw{Gh, Xh, O, I, Kc, gwi ? sGh : nullptr, gwi ? sXh : nullptr, invB, dW, f32, nullptr, ws + L.gws,
                     L.gws_bytes};
    const int kind_x = packed ? 2 : 0, kind_w = gwi ? 0 : 1;
    if (dX && dW && !(flags & HLQ_FLAG_SEPARATE_PRODUCTS) && hlq::gemm_pair_available(kind_x, ax, kind_w, aw))
        return launch_rc(hlq::launch_gemm_pair(kind_x, ax, kind_w, aw, st, defer));
    if (dX && (rc = launch_rc(hlq::launch_gemm_nt(kind_x, ax, st))) != HLQ_OK) return rc;
    if (dW && (rc = launch_rc(hlq::launch_gemm_nt(kind_w, aw, st))) != HLQ_OK) return rc;
    return HLQ_OK;
}

int hlq_linear_backward_mode(const void *G, const void *X, const void *Xc, const float *sXc, const void *W, int64_t N,
                             int64_t d_in, int64_t d_out, int B, int r, uint64_t seed, int dtype, int flags, void *dX,
                             void *dW, void *workspace, size_t workspace_bytes, void *stream)
{
    return backward_impl(G, X, Xc, sXc, W, nullptr, nullptr, N, d_in, d_out, B, r, seed, dtype, flags, dX, dW, workspace,
                         workspace_bytes, stream);
}

int hlq_weight_code_bits(int64_t d_out, int flags)
{
    const int round = (flags & HLQ_FLAG_ROUND_MANTISSA) ? HLQ_BITS_ROUND_MANTISSA : 0;
    if (flags & HLQ_FLAG_GX_8BIT) return HLQ_BITS_8 | round;
    return ((!(flags & HLQ_FLAG_GX_UNPACKED) && d_out % 32 == 0) ? HLQ_BITS_4_PACKED : HLQ_BITS_4) | round;
}

int hlq_linear_backward_cached(const void *G, const void *X, const void *Xc, const float *sXc, const void *WqT,
                               const float *sW, int64_t N, int64_t d_in, int64_t d_out, int B, int r, uint64_t seed,
                               int dtype, int flags, void *dX, void *dW, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    if (dX && (!WqT || !sW)) return HLQ_ERR_NULL;
    return backward_impl(G, X, Xc, sXc, nullptr, dX ? WqT : nullptr, dX ? sW : nullptr, N, d_in, d_out, B, r, seed, dtype,
                         flags, dX, dW, workspace, workspace_bytes, stream);
}

int hlq_linear_backward_ex(const void *G, const void *X, const void *XhatT, const void *W, int64_t N, int64_t d_in,
                           int64_t d_out, int B, int r, uint64_t seed, int dtype, void *dX, void *dW,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    return hlq_linear_backward_mode(G, X, XhatT, nullptr, W, N, d_in, d_out, B, r, seed, dtype, 0, dX, dW, workspace,
                                    workspace_bytes, stream);
}

int hlq_linear_backward(const void *G, const void *X, const void *W, int64_t N, int64_t d_in, int64_t d_out, int B,
                        int r, uint64_t seed, void *dX, void *dW, void *stream)
{
    if (!G || !X || !W || !dX || !dW) return HLQ_ERR_NULL;
    return hlq_linear_backward_ex(G, X, nullptr, W, N, d_in, d_out, B, r, seed, HLQ_BF16, dX, dW, nullptr, 0, stream);
}

// ---- convolution layers (Sec. 3.1) ---------------------------------------------------------------

static int conv_shape(const hlq_conv_geom *g, hlq::ConvShape *out)
{
    if (!g) return HLQ_ERR_NULL;
    if (g->Nb < 1 || g->H < 1 || g->W < 1 || g->C < 1 || g->O < 1 || g->kh < 1 || g->kw < 1 || g->stride_h < 1 ||
        g->stride_w < 1 || g->dil_h < 1 || g->dil_w < 1 || g->pad_h < 0 || g->pad_w < 0)
        return HLQ_ERR_SHAPE;
    const int64_t eh = static_cast<int64_t>(g->H) + 2 * static_cast<int64_t>(g->pad_h) -
                       static_cast<int64_t>(g->dil_h) * (g->kh - 1) - 1;
    const int64_t ew = static_cast<int64_t>(g->W) + 2 * static_cast<int64_t>(g->pad_w) -
                       static_cast<int64_t>(g->dil_w) * (g->kw - 1) - 1;
    if (eh < 0 || ew < 0) return HLQ_ERR_SHAPE;
    const int64_t Ho = eh / g->stride_h + 1, Wo = ew / g->stride_w + 1;
    const int64_t N = g->Nb * Ho * Wo, I = static_cast<int64_t>(g->kh) * g->kw * g->C;
    const int64_t limit = int64_t(1) << 31;
    // the kernels index inside one row of either tensor, and one padded image axis, in 32 bits
    if (N >= limit || I >= limit || static_cast<int64_t>(g->W) * g->C >= limit ||
        static_cast<int64_t>(g->Nb) * g->H >= limit ||
        static_cast<int64_t>(g->H) + 2 * static_cast<int64_t>(g->pad_h) + static_cast<int64_t>(g->kh) * g->dil_h >= limit ||
        static_cast<int64_t>(g->W) + 2 * static_cast<int64_t>(g->pad_w) + static_cast<int64_t>(g->kw) * g->dil_w >= limit)
        return HLQ_ERR_SHAPE;
    hlq::ConvShape c{g->Nb, g->H, g->W, g->C, g->kh, g->kw, g->stride_h, g->stride_w, g->pad_h, g->pad_w,
                     g->dil_h, g->dil_w, static_cast<int>(Ho), static_cast<int>(Wo), N};
    if (out) *out = c;
    return HLQ_OK;
}

static inline bool conv_is_pointwise(const hlq_conv_geom *g)
{
    return g->kh == 1 && g->kw == 1 && g->stride_h == 1 && g->stride_w == 1 && g->pad_h == 0 && g->pad_w == 0;
}

int hlq_conv_sizes(const hlq_conv_geom *g, int64_t *Ho, int64_t *Wo, int64_t *N, int64_t *I)
{
    hlq::ConvShape c;
    const int rc = conv_shape(g, &c);
    if (rc != HLQ_OK) return rc;
    if (Ho) *Ho = c.Ho;
    if (Wo) *Wo = c.Wo;
    if (N) *N = c.N;
    if (I) *I = static_cast<int64_t>(c.kh) * c.kw * c.C;
    return HLQ_OK;
}

int hlq_im2col(const void *X, const hlq_conv_geom *g, int dtype, void *cols, void *stream)
{
    int rc;
    hlq::ConvShape c;
    if (!X || !cols) return HLQ_ERR_NULL;
    if ((rc = conv_shape(g, &c)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if (!aligned(X, 16) || !aligned(cols, 16)) return HLQ_ERR_SHAPE;
    return launch_rc(hlq::launch_im2col(X, c, dtype == HLQ_F32, cols, static_cast<hipStream_t>(stream)));
}

int hlq_col2im(const void *cols, const hlq_conv_geom *g, int dtype, void *dX, void *stream)
{
    int rc;
    hlq::ConvShape c;
    if (!cols || !dX) return HLQ_ERR_NULL;
    if ((rc = conv_shape(g, &c)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if (!aligned(cols, 16) || !aligned(dX, 16)) return HLQ_ERR_SHAPE;
    return launch_rc(hlq::launch_col2im(cols, c, dtype == HLQ_F32, dX, static_cast<hipStream_t>(stream)));
}

static int conv_compress_check(const void *X, const hlq_conv_geom *g, hlq::ConvShape *c, int B, int r, int basis,
                               int dtype)
{
    int rc;
    if ((rc = conv_shape(g, c)) != HLQ_OK) return rc;
    if (!X) return HLQ_ERR_NULL;
    if (basis != HLQ_BASIS_NATURAL && basis != HLQ_BASIS_SEQUENCY) return HLQ_ERR_RANK;
    if ((rc = check_block(B)) != HLQ_OK) return rc;
    if ((rc = check_rank(B, r)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    if ((rc = check_hla_shape(c->N, static_cast<int64_t>(c->kh) * c->kw * c->C, B, r)) != HLQ_OK) return rc;
    if (!hlq::hla_conv_ok(*c, B) || !aligned(X, 16)) return HLQ_ERR_SHAPE;
    return HLQ_OK;
}

int hlq_conv_compress_act(const void *X, const hlq_conv_geom *g, int B, int r, int basis, int dtype, void *XhatT,
                          float *coeffT, void *stream)
{
    int rc;
    hlq::ConvShape c;
    if ((rc = conv_compress_check(X, g, &c, B, r, basis, dtype)) != HLQ_OK) return rc;
    if (!XhatT) return HLQ_ERR_NULL;
    if (!aligned(XhatT, 16) || (coeffT && !aligned(coeffT, 16))) return HLQ_ERR_SHAPE;
    return launch_rc(hlq::launch_hla_conv(X, c, B, r, basis, dtype == HLQ_F32, static_cast<uint16_t *>(XhatT), coeffT,
                                          static_cast<hipStream_t>(stream)));
}

int hlq_conv_compress_act_int8(const void *X, const hlq_conv_geom *g, int B, int r, int basis, uint64_t seed, int dtype,
                               int8_t *XqT, float *sX, float *coeffT, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    int rc;
    hlq::ConvShape c;
    const bool mant = (basis & HLQ_BASIS_ROUND_MANTISSA) != 0;
    basis &= ~HLQ_BASIS_ROUND_MANTISSA;
    if ((rc = conv_compress_check(X, g, &c, B, r, basis, dtype)) != HLQ_OK) return rc;
    if (!XqT || !sX || !workspace) return HLQ_ERR_NULL;
    if (r % 4 != 0) return HLQ_ERR_RANK;
    const int64_t D = static_cast<int64_t>(c.kh) * c.kw * c.C, Kc = c.N / B * r;
    if (Kc % 16 != 0 || D * (Kc / 4) >= (int64_t(1) << 32)) return HLQ_ERR_SHAPE;
    if (!aligned(XqT, 16) || (coeffT && !aligned(coeffT, 16))) return HLQ_ERR_SHAPE;
    if (!aligned(workspace, 256) || workspace_bytes < hlq::hla_quant_ws_bytes(D)) return HLQ_ERR_WORKSPACE;
    const uint64_t key = stream_key(seed, 2);
    return launch_rc(hlq::launch_hla_quant_conv(X, c, B, r, basis, dtype == HLQ_F32, static_cast<uint32_t>(key),
                                                static_cast<uint32_t>(key >> 32), mant, XqT, sX, coeffT, workspace,
                                                static_cast<hipStream_t>(stream)));
}

// Workspace of the convolution pass: [column matrix | column gradient | the linear pass's own].
// The column matrix is stored only when the g_w list cannot read it through the image.
struct ConvLayout {
    bool pointwise, implicit;
    size_t cols, dcols, inner, inner_bytes, total;
};

static ConvLayout conv_layout(const hlq::ConvShape &c, const hlq_conv_geom *g, int B, int r, int dtype, int flags)
{
    const int64_t I = static_cast<int64_t>(c.kh) * c.kw * c.C;
    ConvLayout L;
    L.pointwise = conv_is_pointwise(g);
    L.implicit = !L.pointwise && hlq::hla_conv_ok(c, B);
    const size_t mat = L.pointwise ? 0 : up256(static_cast<size_t>(c.N) * I * (dtype == HLQ_F32 ? 4 : 2));
    L.cols = 0;
    L.dcols = L.implicit ? 0 : mat;
    L.inner = L.dcols + mat;
    L.inner_bytes = hlq_workspace_bytes_mode(c.N, I, g->O, B, r, 0, flags);
    L.total = L.inner + L.inner_bytes;
    return L;
}

size_t hlq_conv_workspace_bytes(const hlq_conv_geom *g, int B, int r, int dtype, int flags)
{
    hlq::ConvShape c;
    if (conv_shape(g, &c) != HLQ_OK || check_dtype(dtype) != HLQ_OK || check_block(B) != HLQ_OK) return 0;
    const ConvLayout L = conv_layout(c, g, B, r, dtype, flags);
    return L.inner_bytes == 0 ? 0 : L.total;
}

int hlq_conv2d_backward(const void *G, const void *X, const void *Wt, const hlq_conv_geom *g, int B, int r,
                        uint64_t seed, int dtype, int flags, void *dX, void *dW, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    int rc;
    hlq::ConvShape c;
    if ((rc = conv_shape(g, &c)) != HLQ_OK) return rc;
    if ((rc = check_dtype(dtype)) != HLQ_OK) return rc;
    const int64_t I = static_cast<int64_t>(c.kh) * c.kw * c.C;
    // every refusal of the linear pass, before anything is launched (the image stands in for the
    // column matrix; the buffers inside the workspace are aligned by construction)
    if ((rc = backward_check(G, dW ? X : nullptr, nullptr, nullptr, dX ? Wt : nullptr, nullptr, nullptr, c.N, I, g->O, B,
                             r, dtype, flags, dX, dW)) != HLQ_OK)
        return rc;
    const ConvLayout L = conv_layout(c, g, B, r, dtype, flags);
    char *ws = static_cast<char *>(workspace);
    if (ws) {
        if (!aligned(ws, 256) || workspace_bytes < L.total) return HLQ_ERR_WORKSPACE;
    } else {
        void *p = nullptr;
        if ((rc = own_workspace(L.total, &p)) != HLQ_OK) return rc;
        ws = static_cast<char *>(p);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool f32 = dtype == HLQ_F32;
    const void *xmat = X;
    void *dxmat = dX;
    if (!L.pointwise) {
        if (dW && !L.implicit) {
            if ((rc = launch_rc(hlq::launch_im2col(X, c, f32, ws + L.cols, st))) != HLQ_OK) return rc;
            xmat = ws + L.cols;
        }
        if (dX) dxmat = ws + L.dcols;
    }
    const bool fold = !L.pointwise && dX;
    hlq::SplitReduce red{};
    rc = backward_impl(G, dW ? xmat : nullptr, nullptr, nullptr, dX ? Wt : nullptr, nullptr, nullptr, c.N, I, g->O, B, r,
                       seed, dtype, flags, dxmat, dW, ws + L.inner, L.inner_bytes, stream, L.implicit ? &c : nullptr,
                       fold ? &red : nullptr);
    if (rc != HLQ_OK) return rc;
    // the fold, and in the same launch the reduction that the weight gradient's product left to do, if any
    if (fold) return launch_rc(hlq::launch_col2im(dxmat, c, f32, dX, st, &red));
    return HLQ_OK;
}

}  // extern "C"
