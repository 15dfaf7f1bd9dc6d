// K2 | K4 as one persistent launch (gemm_stream_body.hpp): one workgroup per compute unit walks its
// share of the tiles of the g_x product (arXiv 2406.15102, Sec. 6.1, stages 5-6), then its share of
// the g_w product's (stage 5).  Used for layers whose products are several 256 x 256 tiles per
// compute unit; everything else keeps one workgroup per tile (k_gemm.hip, k_gemm_pair.hip).
#include "gemm_plan.hpp"
#include "gemm_stream_body.hpp"

#include <atomic>
#include <mutex>

namespace hlq {

template <int KA, int KB>
__global__ __launch_bounds__(256) void k_gemm_stream(GemmDev ga, GemmDev gb)
{
    const int wg = static_cast<int>(blockIdx.x), nwg = static_cast<int>(gridDim.x);
    if (ga.tiles_m > 0) gemm_stream_product<KA>(ga, wg, nwg);
    if (gb.tiles_m > 0) gemm_stream_product<KB>(gb, wg, nwg);
}

namespace {
// Off by default: the tile-per-workgroup kernels that load their operands straight into LDS
// (gemm_dl_body.hpp) are ahead of this form wherever it applies -- 8192 x 28672 x 8192, both products,
// same session: 2150 us one workgroup per tile through registers, 2143 persistent, 2075 straight into
// LDS -- and the ring of that body leaves no LDS for an epilogue that overlaps the next tile's loads.
std::atomic<int> g_stream_enabled{0};

// compute units of the current device, rounded down to a multiple of 8 (one workgroup each; the
// tile lists are cut per XCD); 0 if unknown
int stream_grid()
{
    static std::mutex mtx;
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return 0;
    }
    std::lock_guard<std::mutex> lock(mtx);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
            (void)hipGetLastError();
            n = 0;
        }
        cached[dev] = n >= 8 ? (n / 8) * 8 : -1;
    }
    return cached[dev] > 0 ? cached[dev] : 0;
}

bool product_ok(int kind, const GemmArgs &a)
{
    const int Kb = row_bytes(kind, a.K);
    return a.C && !a.acc && !a.c_is_f32 && Kb % 128 == 0 && Kb / 128 >= 4 && a.M > 0 && a.N > 0;
}

int tiles256(const GemmArgs &a) { return ((a.M + 255) / 256) * ((a.N + 255) / 256); }

template <int KA, int KB>
hipError_t launch_tt(const GemmDev &ga, const GemmDev &gb, int grid, hipStream_t st)
{
    constexpr size_t lds_bytes = gemm_stream_lds_bytes();
    static bool attr_set = false;     // idempotent; racing callers set the same value
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_stream<KA, KB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_gemm_stream<KA, KB>), dim3(grid), dim3(256), lds_bytes, st, ga, gb);
    return hipGetLastError();
}
}  // namespace

void gemm_stream_enable(bool on) { g_stream_enabled.store(on ? 1 : 0); }

// a: the g_x product or the only one; b: the g_w product or NULL
bool gemm_stream_wanted(int kindA, const GemmArgs &a, int kindB, const GemmArgs *b)
{
    if (!g_stream_enabled.load()) return false;
    if (!product_ok(kindA, a) || (b && !product_ok(kindB, *b))) return false;
    if (!(kindA == 0 || kindA == 1 || kindA == 2) || (b && !(kindB == 0 || kindB == 1))) return false;
    const int grid = stream_grid();
    if (grid == 0) return false;
    // Measured on MI355X against one workgroup per tile (same session, alternating): at 3.7 tiles per
    // compute unit (4096 x 4096 x 11008) the two forms take the same time within 1 %, either way;
    // at 28 tiles per compute unit (8192 x 28672 x 8192) the persistent form is 0.8 % (both products)
    // to 1.8 % (the g_x product alone) faster.  When switched on it is used from four tiles per compute unit on.
    return tiles256(a) + (b ? tiles256(*b) : 0) >= 4 * grid;
}

hipError_t launch_gemm_stream(int kindA, const GemmArgs &a, int kindB, const GemmArgs *b, hipStream_t st)
{
    const int grid = stream_grid();
    if (grid == 0) return hipErrorInvalidValue;
    const GemmDev ga = gemm_dev(kindA, a, 256, 256, 1);
    GemmDev gb{};
    if (b) gb = gemm_dev(kindB, *b, 256, 256, 1);
    if (!b) {
        switch (kindA) {
            case 0: return launch_tt<0, 0>(ga, gb, grid, st);
            case 1: return launch_tt<1, 1>(ga, gb, grid, st);
            default: return launch_tt<2, 1>(ga, gb, grid, st);
        }
    }
    if (kindA == 2) return kindB == 1 ? launch_tt<2, 1>(ga, gb, grid, st) : launch_tt<2, 0>(ga, gb, grid, st);
    return kindB == 1 ? launch_tt<0, 1>(ga, gb, grid, st) : launch_tt<0, 0>(ga, gb, grid, st);
}

}  // namespace hlq
