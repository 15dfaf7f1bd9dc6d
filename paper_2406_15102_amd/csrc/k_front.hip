// The transforms of one backward pass, launched together.  Stages 1-2 of the g_x list (K1 on G),
// stages 1 and 3 of the g_w list (K3 on X and on G) and the first pass of stages 3-4 of the g_x
// list (column maxima of H^T W) do not depend on one another (arXiv 2406.15102, Sec. 6.1), and each
// costs a few tens of microseconds, of which four to five are the fixed price of a launch that
// waits for its predecessor to drain.  Two launches carry them instead of six:
//   front A   K1(G)  |  K3(G)  |  K3(X)  |  zeroing of the column maxima    (workgroups of the quantiser and of
//                                                                           the projections in turns)
//   front B   column maxima of H^T W                                        (needs the zeroing)
// (with HLQ_OPT_FRONT_INTERLEAVE off, each job keeps its own index range and K3(X) rides in front B; a
// convolution has K3 of the image, read as its column matrix, in front A and K3(G) in front B)
// or ONE, when the weight has few row blocks (k_front_one below): the maxima stay per row block.
// and three launches carry the integer g_w list, whose projections are quantised in two passes too:
//   front A   K1(G)  |  zeroing of all three sets of maxima
//   front Q1  maxima of projected G  |  of projected X  |  of H^T W
//   front Q2  int8 codes of projected G  |  of projected X  |  codes of the weight
// A workgroup looks up its job from its index (jobs occupy consecutive index ranges, a job may be
// empty) and runs the same device body as the stand-alone kernel of that stage.
#include "hla_body.hpp"
#include "hlq_kernels.hpp"
#include "quant_cols_body.hpp"
#include "quant_rows_body.hpp"

#include <atomic>

namespace hlq {

FrontMix front_mix_of(int n1, int n3);

// Workgroup b of the n1 + n3 that two kinds of job share, handed out in turns (FrontMix): k1 >= 0, the index
// among the first kind, or k3 >= 0, among the second; both < 0 past the end, with b counted from there.
__device__ __forceinline__ void front_turns(const FrontMix &jm, int &b, int n1, int n3, int &k1, int &k3)
{
    const int per = jm.gran * (jm.q + 1);
    k1 = k3 = -1;
    if (b < jm.cyc * per) {
        const int turn = b / per, pos = b % per;
        if (pos < jm.gran * jm.q) k1 = turn * jm.gran * jm.q + pos;
        else k3 = turn * jm.gran + pos - jm.gran * jm.q;
        return;
    }
    b -= jm.cyc * per;
    const int k1_left = n1 - jm.cyc * jm.gran * jm.q, k3_left = n3 - jm.cyc * jm.gran;
    if (b < k1_left) k1 = jm.cyc * jm.gran * jm.q + b;
    else if (b - k1_left < k3_left) k3 = jm.cyc * jm.gran + b - k1_left;
    else b -= k1_left + k3_left;
}

// CONV: X is a channels-last image and K3 reads its column matrix through ConvRows.  A kernel of
// its own: the extra address arithmetic would cost the matrix variant registers, and with them a
// wavefront of occupancy at B = 32.
template <typename Tin, int B, bool PACKED, int BASIS, bool CONV>
__global__ __launch_bounds__(256) void k_front_a(FrontRows jr, FrontHla jx, FrontFill jf, FrontConv jc, FrontShare js,
                                                 FrontMix jm, FrontHla jy)
{
    int b = blockIdx.x;
    if (!CONV && js.on) {
        // K1 and K3 read the same tensor: both readers of a group of 128 rows on one XCD, one after the other
        if (b < js.blocks) {
            const int per = js.nk1 + js.gx;
            const int xcd = b & 7, q = b >> 3;
            const int unit = (q / (js.pair * per)) * 8 + xcd;
            const int u = q % (js.pair * per);
            const int grp = unit * js.pair + u / per, v = u % per;
            if (unit >= js.units) return;
            if (v < js.nk1) {
                const int blk = grp * js.nk1 + v;
                if (blk < jr.blocks)
                    quant_rows_body<Tin, B, 256, PACKED>(static_cast<const Tin *>(jr.G), jr.N, jr.O, jr.T, jr.k0, jr.k1, jr.qmax,
                                                         jr.Gq, jr.sG, nullptr, blk);
            } else {
                hla_body<Tin, B, BASIS, 2>(static_cast<const Tin *>(jx.T), jx.N, jx.D, jx.r, jx.out, nullptr, v - js.nk1, grp);
            }
            return;
        }
        b -= js.blocks;
        const int i = b * 256 + threadIdx.x;
        if (i < jf.n) jf.p[i] = 0u;
        return;
    }
    if (!CONV && jm.gran) {
        int k1, k3;
        front_turns(jm, b, jr.blocks, jx.nb + jy.nb, k1, k3);
        if (k1 >= 0) {
            quant_rows_body<Tin, B, 256, PACKED>(static_cast<const Tin *>(jr.G), jr.N, jr.O, jr.T, jr.k0, jr.k1, jr.qmax, jr.Gq,
                                                 jr.sG, nullptr, k1);
        } else if (k3 >= 0 && k3 < jx.nb) {
            int bx, by;
            hla_job_map(k3, jx.gx, jx.grp, bx, by);
            hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jx.T), jx.N, jx.D, jx.r, jx.out, nullptr, bx, by);
        } else if (k3 >= 0) {
            int bx, by;
            hla_job_map(k3 - jx.nb, jy.gx, jy.grp, bx, by);
            hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jy.T), jy.N, jy.D, jy.r, jy.out, nullptr, bx, by);
        } else {
            const int i = b * 256 + threadIdx.x;
            if (i < jf.n) jf.p[i] = 0u;
        }
        return;
    }
    if (b < jr.blocks) {
        quant_rows_body<Tin, B, 256, PACKED>(static_cast<const Tin *>(jr.G), jr.N, jr.O, jr.T, jr.k0, jr.k1, jr.qmax, jr.Gq,
                                             jr.sG, nullptr, b);
        return;
    }
    b -= jr.blocks;
    if (b < jx.nb) {
        int bx, by;
        hla_job_map(b, jx.gx, jx.grp, bx, by);
        if (CONV)
            hla_body_src<B, BASIS>(ConvRows<Tin>{static_cast<const Tin *>(jx.T), jc.g}, jx.N, jx.D, jx.r, jx.out, nullptr, bx, by);
        else
            hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jx.T), jx.N, jx.D, jx.r, jx.out, nullptr, bx, by);
        return;
    }
    b -= jx.nb;
    if (b < jy.nb) {
        int bx, by;
        hla_job_map(b, jy.gx, jy.grp, bx, by);
        hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jy.T), jy.N, jy.D, jy.r, jy.out, nullptr, bx, by);
        return;
    }
    b -= jy.nb;
    const int i = b * 256 + threadIdx.x;
    if (i < jf.n) jf.p[i] = 0u;
}

// The whole front in one launch, for weights of few rows: a workgroup per strip of columns runs both
// passes of K1T (cols_full_body), so neither a zeroing launch before it nor a launch for pass 2 is needed.
// (three wavefronts per SIMD asked for below B = 64, which the other jobs had before the strip quantiser
// joined them: left alone, the register allocator spends all 256 registers on it)
template <typename Tin, int B, bool PACKED, int BASIS, bool CONV>
__global__ __launch_bounds__(256, B == 64 ? 2 : 3) void k_front_one(FrontRows jr, FrontHla jx, FrontHla jg, FrontColsQ jq, FrontConv jc,
                                                                    FrontMix jm)
{
    int b = blockIdx.x;
    if (b < jq.gx) {       // first: these workgroups pass over their strip twice
        cols_full_body<Tin, B, PACKED>(static_cast<const Tin *>(jq.W), jq.O, jq.I, jq.k0, jq.k1, jq.qmax, jq.WqT, jq.sW, b, jq.gy);
        return;
    }
    b -= jq.gx;
    if (jm.gran) {
        // the row quantiser's workgroups and the projections' in turns: b becomes an index in the ranges below
        int k1, k3;
        front_turns(jm, b, jr.blocks, jx.nb + jg.nb, k1, k3);
        if (k1 < 0 && k3 < 0) return;
        b = k1 >= 0 ? k1 : jr.blocks + k3;
    }
    if (b < jr.blocks) {
        quant_rows_body<Tin, B, 256, PACKED>(static_cast<const Tin *>(jr.G), jr.N, jr.O, jr.T, jr.k0, jr.k1, jr.qmax, jr.Gq,
                                             jr.sG, nullptr, b);
        return;
    }
    b -= jr.blocks;
    if (b < jx.nb) {
        int bx, by;
        hla_job_map(b, jx.gx, jx.grp, bx, by);
        if (CONV)
            hla_body_src<B, BASIS>(ConvRows<Tin>{static_cast<const Tin *>(jx.T), jc.g}, jx.N, jx.D, jx.r, jx.out, nullptr, bx, by);
        else
            hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jx.T), jx.N, jx.D, jx.r, jx.out, nullptr, bx, by);
        return;
    }
    b -= jx.nb;
    int bx, by;
    hla_job_map(b, jg.gx, jg.grp, bx, by);
    hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jg.T), jg.N, jg.D, jg.r, jg.out, nullptr, bx, by);
}

template <typename Tin, int B, int BASIS>
__global__ __launch_bounds__(256) void k_front_b(FrontHla jg, FrontAbsmax jw)
{
    int b = blockIdx.x;
    if (b < jg.nb) {
        int bx, by;
        hla_job_map(b, jg.gx, jg.grp, bx, by);
        hla_body<Tin, B, BASIS>(static_cast<const Tin *>(jg.T), jg.N, jg.D, jg.r, jg.out, nullptr, bx, by);
        return;
    }
    b -= jg.nb;
    cols_absmax_body<Tin, B>(static_cast<const Tin *>(jw.W), jw.O, jw.I, jw.amax, b % jw.gx, b / jw.gx);
}

// integer g_w list, pass 1 of everything: maxima of the kept coefficients of G and of X, of H^T W
// With jr (the row quantiser of G, which waits for nothing) riding along, in turns: its arithmetic beside three
// passes that only read.
template <typename Tin, int B, int BASIS, bool PACKED>
__global__ __launch_bounds__(256) void k_front_q1(FrontHlaQ jg, FrontHlaQ jx, FrontAbsmax jw, FrontRows jr, FrontMix jm)
{
    int b = blockIdx.x;
    if (jr.blocks > 0) {
        int k1 = -1, k3 = -1;
        const int n3 = jg.gx * jg.gy + jx.gx * jx.gy + jw.gx * jw.gy;
        if (jm.gran) {
            front_turns(jm, b, jr.blocks, n3, k1, k3);
        } else if (b < jr.blocks) {
            k1 = b;
        } else {
            k3 = b - jr.blocks;
        }
        if (k1 >= 0) {
            quant_rows_body<Tin, B, 256, PACKED>(static_cast<const Tin *>(jr.G), jr.N, jr.O, jr.T, jr.k0, jr.k1, jr.qmax, jr.Gq,
                                                 jr.sG, nullptr, k1);
            return;
        }
        if (k3 < 0) return;
        b = k3;
    }
    if (b < jg.gx * jg.gy) {
        hla_absmax_body<Tin, B, BASIS>(static_cast<const Tin *>(jg.T), jg.N, jg.D, jg.r, jg.amax, b % jg.gx, b / jg.gx);
        return;
    }
    b -= jg.gx * jg.gy;
    if (b < jx.gx * jx.gy) {
        hla_absmax_body<Tin, B, BASIS>(static_cast<const Tin *>(jx.T), jx.N, jx.D, jx.r, jx.amax, b % jx.gx, b / jx.gx);
        return;
    }
    b -= jx.gx * jx.gy;
    cols_absmax_body<Tin, B>(static_cast<const Tin *>(jw.W), jw.O, jw.I, jw.amax, b % jw.gx, b / jw.gx);
}

// pass 2 of everything: int8 codes of projected G and X, codes of the weight
template <typename Tin, int B, int BASIS, bool PACKED>
__global__ __launch_bounds__(256) void k_front_q2(FrontHlaQ jg, FrontHlaQ jx, FrontColsQ jq)
{
    // backwards through the jobs and through each of them (reverse_same_xcd): what the passes that took the maxima
    // read last is what the last-level cache still holds
    const int64_t bytes = (jg.T ? jg.N * jg.D : 0) + (jx.T ? jx.N * jx.D : 0) + (jq.W ? static_cast<int64_t>(jq.O) * jq.I : 0);
    int b = reverse_same_xcd(blockIdx.x, gridDim.x, bytes * static_cast<int64_t>(sizeof(Tin)));
    if (b < jg.gx * jg.gy) {
        hla_quantize_body<Tin, B, BASIS>(static_cast<const Tin *>(jg.T), jg.N, jg.D, jg.r, jg.amax, jg.k0, jg.k1, jg.TqT,
                                         jg.sT, nullptr, b % jg.gx, b / jg.gx);
        return;
    }
    b -= jg.gx * jg.gy;
    if (b < jx.gx * jx.gy) {
        hla_quantize_body<Tin, B, BASIS>(static_cast<const Tin *>(jx.T), jx.N, jx.D, jx.r, jx.amax, jx.k0, jx.k1, jx.TqT,
                                         jx.sT, nullptr, b % jx.gx, b / jx.gx);
        return;
    }
    b -= jx.gx * jx.gy;
    cols_quantize_body<Tin, B, PACKED>(static_cast<const Tin *>(jq.W), jq.O, jq.I, jq.amax, jq.k0, jq.k1, jq.qmax, jq.WqT,
                                       jq.sW, nullptr, b % jq.gx, b / jq.gx);
}

FrontHlaQ front_hlaq(const void *T, int64_t N, int D, int B, int r, uint32_t *amax, uint32_t k0, uint32_t k1, int8_t *TqT,
                     float *sT)
{
    FrontHlaQ j{T, N, D, r, amax, k0, k1, TqT, sT, 0, 0};
    if (!T) return j;
    j.gx = hla_grid_x(D, B);
    j.gy = hla_grid_y(N, B);
    return j;
}

FrontColsQ front_colsq(const void *W, int O, int I, int B, const uint32_t *amax, uint32_t k0, uint32_t k1, float qmax,
                       int8_t *WqT, float *sW)
{
    FrontColsQ j{W, O, I, amax, k0, k1, qmax, WqT, sW, 0, 0};
    if (!W) return j;
    j.gx = cols_grid_x(I, B);
    j.gy = cols_grid_y(O, B);
    return j;
}

template <typename Tin, int B, int BASIS>
static hipError_t launch_front_q_t(const FrontHlaQ &jg, const FrontHlaQ &jx, const FrontAbsmax &jw, const FrontColsQ &jq,
                                   const FrontRows &jr, bool packed, hipStream_t st)
{
    const int n3 = jg.gx * jg.gy + jx.gx * jx.gy + jw.gx * jw.gy;
    const int n1 = n3 + jr.blocks;
    const FrontMix jm = jr.blocks > 0 ? front_mix_of(jr.blocks, n3) : FrontMix{0, 0, 0};
    if (n1 > 0) {
        if (packed) hipLaunchKernelGGL((k_front_q1<Tin, B, BASIS, true>), dim3(n1), dim3(256), 0, st, jg, jx, jw, jr, jm);
        else hipLaunchKernelGGL((k_front_q1<Tin, B, BASIS, false>), dim3(n1), dim3(256), 0, st, jg, jx, jw, jr, jm);
    }
    const int n2 = jg.gx * jg.gy + jx.gx * jx.gy + jq.gx * jq.gy;
    if (n2 > 0) {
        if (packed) hipLaunchKernelGGL((k_front_q2<Tin, B, BASIS, true>), dim3(n2), dim3(256), 0, st, jg, jx, jq);
        else hipLaunchKernelGGL((k_front_q2<Tin, B, BASIS, false>), dim3(n2), dim3(256), 0, st, jg, jx, jq);
    }
    return hipGetLastError();
}

hipError_t launch_front_q(const FrontHlaQ &jg, const FrontHlaQ &jx, const FrontAbsmax &jw, const FrontColsQ &jq,
                          const FrontRows &jr, int B, int basis, bool is_f32, bool packed, hipStream_t st)
{
#define HLQ_FRONTQ_CASE(BB)                                                                     \
    case BB:                                                                                    \
        if (basis)                                                                              \
            return is_f32 ? launch_front_q_t<float, BB, 1>(jg, jx, jw, jq, jr, packed, st)          \
                          : launch_front_q_t<bf16_t, BB, 1>(jg, jx, jw, jq, jr, packed, st);        \
        return is_f32 ? launch_front_q_t<float, BB, 0>(jg, jx, jw, jq, jr, packed, st)              \
                      : launch_front_q_t<bf16_t, BB, 0>(jg, jx, jw, jq, jr, packed, st);
    switch (B) {
        HLQ_FRONTQ_CASE(16)
        HLQ_FRONTQ_CASE(32)
        HLQ_FRONTQ_CASE(64)
    }
#undef HLQ_FRONTQ_CASE
    return hipErrorInvalidValue;
}

bool front_fusable(int O, int B)
{
    const int T = quant_rows_lanes(O, B);
    return T > 0;   // rows that need the 1024-thread K1 keep their own launch
}

FrontRows front_rows(const void *G, int64_t N, int O, int B, uint32_t k0, uint32_t k1, float qmax, int8_t *Gq, float *sG)
{
    FrontRows j{G, N, O, 0, k0, k1, qmax, Gq, sG, 0};
    if (!G) return j;
    j.T = quant_rows_lanes(O, B);
    const int rows_per_block = 256 / j.T;     // T == 256: one row per workgroup
    j.blocks = static_cast<int>((N + rows_per_block - 1) / rows_per_block);
    return j;
}

FrontHla front_hla(const void *T, int64_t N, int D, int B, int r, uint16_t *out)
{
    FrontHla j{T, N, D, r, out, 0, 0, 1, 0};
    if (!T) return j;
    j.gx = hla_grid_x(D, B);
    j.gy = hla_grid_y(N, B);
    j.grp = hla_job_grp(B, r);
    j.nb = hla_job_blocks(j.gx, j.gy, j.grp);
    return j;
}

FrontAbsmax front_absmax(const void *W, int O, int I, int B, uint32_t *amax)
{
    FrontAbsmax j{W, O, I, amax, 0, 0};
    if (!W) return j;
    j.gx = cols_grid_x(I, B);
    j.gy = cols_grid_y(O, B);
    return j;
}

bool cols_full_ok(int O, int I, int B, bool is_f32)
{
    return O / B <= kColsFullMaxRowBlocks && static_cast<int64_t>(O) * I * (is_f32 ? 4 : 2) <= kColsFullMaxBytes;
}

FrontColsQ front_cols_full(const void *W, int O, int I, int B, uint32_t k0, uint32_t k1, float qmax, int8_t *WqT, float *sW)
{
    FrontColsQ j{W, O, I, nullptr, k0, k1, qmax, WqT, sW, 0, 0};
    if (!W) return j;
    // as many groups of lanes as there are row blocks, so that a pass is one round where it can be: 16, 32 or
    // 64; beyond 64 row blocks there are several rounds anyway and the longer runs of 32 groups measure better
    const int nrb = O / B;
    const int lg = nrb <= 16 ? 4 : (nrb <= 32 ? 3 : (nrb <= 64 ? 2 : 3));
    const int strip = (B == 16 ? ColsFull<16>::CW : (B == 32 ? ColsFull<32>::CW : ColsFull<64>::CW)) << lg;
    j.gx = (I + strip - 1) / strip;
    j.gy = lg;
    return j;
}

namespace {
// Off by default.  Measured at 4096 x 4096 x 11008 (rocprofv3, 212 launches each way): with the shared
// read the launch fetches 98.5 MB instead of 180.6 MB from beyond the L2s -- G comes in once -- and
// takes 51.5 us instead of 53.0, the whole pass the same either way: the launch is bound by the
// quantiser's arithmetic and by latency, not by those bytes (its second read of G is served by the
// last-level cache).  A first form with groups of 64 rows and narrower K3 workgroups, whose write
// runs were shorter, took 62.4 us.
std::atomic<int> g_share_enabled{0};
}
void front_share_enable(bool on) { g_share_enabled.store(on ? 1 : 0); }

namespace {
// On by default.  Whole pass at 4096 x 4096 x 11008, alternating runs on one box: 371.9 us with each job in its
// own range, 364-367 with turns of 8 to 128 workgroups of the projection (32 the best by a microsecond);
// 8192 x 28672 x 8192 and the small layers do not move.
std::atomic<int> g_mix_enabled{1};
constexpr int kMixGran = 32;     // a multiple of 8: hla_job_map counts on index mod 8 being the XCD
}
void front_mix_enable(bool on) { g_mix_enabled.store(on ? 1 : 0); }
bool front_mix_enabled() { return g_mix_enabled.load() != 0; }

// turns for n1 workgroups of the quantiser and n3 of the projections; gran == 0 if either has too few
FrontMix front_mix_of(int n1, int n3)
{
    FrontMix m{0, 0, 0};
    if (!g_mix_enabled.load() || n1 < kMixGran || n3 < kMixGran) return m;
    m.gran = kMixGran;
    m.q = (n1 + n3 / 2) / n3;     // workgroups of the quantiser per workgroup of the projections
    if (m.q < 1) m.q = 1;
    const int c1 = n1 / (m.gran * m.q), c3 = n3 / m.gran;
    m.cyc = c1 < c3 ? c1 : c3;
    if (m.cyc == 0) m.gran = 0;
    return m;
}

FrontMix front_mix(const FrontRows &jr, const FrontHla &jx, int more)
{
    if (!jr.G || !jx.T) return FrontMix{0, 0, 0};
    return front_mix_of(jr.blocks, jx.nb + more);
}

FrontShare front_share(const FrontRows &jr, const FrontHla &jx, int B, bool is_f32)
{
    FrontShare s{};
    if (!g_share_enabled.load() || !jr.G || jr.G != jx.T || jr.N != jx.N || jr.O != jx.D) return s;
    constexpr int RG = 128;                             // rows of a group: 128 / B token blocks of K3
    const int rows_per_k1 = 256 / jr.T;                 // T = 256: one row per workgroup
    if (RG % rows_per_k1 != 0) return s;
    // Only where it pays: a group's rows (and what is written for them) must sit in one XCD's L2
    // together (4 MB), and the tensor must be large enough for its second read to cost real time.
    const int64_t row_bytes = static_cast<int64_t>(jr.O) * (is_f32 ? 4 : 2);
    if (row_bytes * RG > (int64_t(3) << 20) || row_bytes * jr.N < (int64_t(16) << 20)) return s;
    const int64_t groups = (jr.N + RG - 1) / RG;
    int pair = B / (2 * jx.r);                          // K3 writes 256 r / B bytes per column and group
    if (pair < 1) pair = 1;
    if (pair > 8) pair = 8;
    const int64_t units = (groups + pair - 1) / pair;
    s.nk1 = RG / rows_per_k1;
    s.gx = (jr.O + 255) / 256;
    s.pair = pair;
    const int64_t blocks = 8 * ((units + 7) / 8) * pair * (s.nk1 + s.gx);
    if (blocks >= (int64_t(1) << 30)) return FrontShare{};
    s.units = static_cast<int>(units);
    s.blocks = static_cast<int>(blocks);
    s.on = 1;
    return s;
}

template <typename Tin, int B, int BASIS>
static hipError_t launch_front_t(const FrontRows &jr, const FrontHla &jx, const FrontFill &jf, const FrontHla &jg,
                                 const FrontAbsmax &jw, const FrontConv &jc, bool packed, hipStream_t st)
{
    const FrontShare js = jc.on ? FrontShare{} : front_share(jr, jx, B, sizeof(Tin) == 4);
    // Unless that is switched off, the first launch takes both projections (the second is left with the pass
    // over W, if there is one) and hands out its workgroups in turns: the row quantiser's arithmetic then has
    // all the memory-bound work there is to run beside.
    const FrontHla none = front_hla(nullptr, 0, 0, B, 1, nullptr);
    const bool both = g_mix_enabled.load() && !jc.on && !js.on && jg.T;
    const FrontMix jm = (jc.on || js.on) ? FrontMix{0, 0, 0} : front_mix(jr, jx, both ? jg.nb : 0);
    const FrontHla &jy = both ? jg : none;        // second projection of the first launch
    const FrontHla &jb = both ? none : jg;        // projection of the second launch
    const int na = (js.on ? js.blocks : jr.blocks + jx.nb + jy.nb) + (jf.n + 255) / 256;
    if (na > 0) {
#define HLQ_FRONT_A(P, CV) hipLaunchKernelGGL((k_front_a<Tin, B, P, BASIS, CV>), dim3(na), dim3(256), 0, st, jr, jx, jf, jc, js, jm, jy)
        if (jc.on) {
            if (packed) HLQ_FRONT_A(true, true); else HLQ_FRONT_A(false, true);
        } else {
            if (packed) HLQ_FRONT_A(true, false); else HLQ_FRONT_A(false, false);
        }
#undef HLQ_FRONT_A
    }
    const int nb = jb.nb + jw.gx * jw.gy;
    if (nb > 0) hipLaunchKernelGGL((k_front_b<Tin, B, BASIS>), dim3(nb), dim3(256), 0, st, jb, jw);
    return hipGetLastError();
}

template <typename Tin, int B, int BASIS>
static hipError_t launch_front_one_t(const FrontRows &jr, const FrontHla &jx, const FrontHla &jg, const FrontColsQ &jq,
                                     const FrontConv &jc, bool packed, hipStream_t st)
{
    const int n = jq.gx + jr.blocks + jx.nb + jg.nb;
    if (n == 0) return hipSuccess;
    // (layers whose quantiser has fewer than a thousand workgroups lose a little by it: 29.3 -> 30.0 us at 12544 x 896 x 224)
    const FrontMix jm = (jr.G && jr.blocks >= 1024) ? front_mix_of(jr.blocks, jx.nb + jg.nb) : FrontMix{0, 0, 0};
#define HLQ_FRONT_ONE(P, CV) hipLaunchKernelGGL((k_front_one<Tin, B, P, BASIS, CV>), dim3(n), dim3(256), 0, st, jr, jx, jg, jq, jc, jm)
    if (jc.on) {
        if (packed) HLQ_FRONT_ONE(true, true); else HLQ_FRONT_ONE(false, true);
    } else {
        if (packed) HLQ_FRONT_ONE(true, false); else HLQ_FRONT_ONE(false, false);
    }
#undef HLQ_FRONT_ONE
    return hipGetLastError();
}

hipError_t launch_front_one(const FrontRows &jr, const FrontHla &jx, const FrontHla &jg, const FrontColsQ &jq,
                            const ConvShape *conv, int B, int basis, bool is_f32, bool packed, hipStream_t st)
{
    FrontConv jc{};
    if (conv) {
        if (!hla_conv_ok(*conv, B)) return hipErrorInvalidValue;
        jc.g = *conv;
        jc.on = 1;
    }
    if (jq.W && (jq.O / B > kColsFullMaxRowBlocks || jq.gy < 2 || jq.gy > 4)) return hipErrorInvalidValue;
#define HLQ_FRONT1_CASE(BB)                                                                     \
    case BB:                                                                                    \
        if (basis)                                                                              \
            return is_f32 ? launch_front_one_t<float, BB, 1>(jr, jx, jg, jq, jc, packed, st)    \
                          : launch_front_one_t<bf16_t, BB, 1>(jr, jx, jg, jq, jc, packed, st);  \
        return is_f32 ? launch_front_one_t<float, BB, 0>(jr, jx, jg, jq, jc, packed, st)        \
                      : launch_front_one_t<bf16_t, BB, 0>(jr, jx, jg, jq, jc, packed, st);
    switch (B) {
        HLQ_FRONT1_CASE(16)
        HLQ_FRONT1_CASE(32)
        HLQ_FRONT1_CASE(64)
    }
#undef HLQ_FRONT1_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_front(const FrontRows &jr, const FrontHla &jx, const FrontFill &jf, const FrontHla &jg,
                        const FrontAbsmax &jw, const ConvShape *conv, int B, int basis, bool is_f32, bool packed,
                        hipStream_t st)
{
    FrontConv jc{};
    if (conv) {
        if (!hla_conv_ok(*conv, B)) return hipErrorInvalidValue;
        jc.g = *conv;
        jc.on = 1;
    }
#define HLQ_FRONT_CASE(BB)                                                                      \
    case BB:                                                                                    \
        if (basis)                                                                              \
            return is_f32 ? launch_front_t<float, BB, 1>(jr, jx, jf, jg, jw, jc, packed, st)        \
                          : launch_front_t<bf16_t, BB, 1>(jr, jx, jf, jg, jw, jc, packed, st);      \
        return is_f32 ? launch_front_t<float, BB, 0>(jr, jx, jf, jg, jw, jc, packed, st)            \
                      : launch_front_t<bf16_t, BB, 0>(jr, jx, jf, jg, jw, jc, packed, st);
    switch (B) {
        HLQ_FRONT_CASE(16)
        HLQ_FRONT_CASE(32)
        HLQ_FRONT_CASE(64)
    }
#undef HLQ_FRONT_CASE
    return hipErrorInvalidValue;
}

}  // namespace hlq
