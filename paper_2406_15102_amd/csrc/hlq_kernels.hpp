// Host-side launchers of the gfx950 kernels.  Every launcher only enqueues work on `st`; shapes
// have been validated by the caller (hlq_api.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hlq {

// K1: rows of G -> codes + per-row scales (and optionally the fp32 coefficients).  `packed`
// (4-bit codes only): two codes to a byte, O/2 bytes per row, instead of one int8 each.
// `mant`: round by the low 11 mantissa bits of each value instead of the seeded stream (k0, k1 unused).
hipError_t launch_quant_rows(const void *G, int64_t N, int O, int B, bool is_f32, uint32_t k0, uint32_t k1,
                             float qmax, bool packed, bool mant, int8_t *Gq, float *sG, float *coeff, hipStream_t st);

// K1T: W [O, I] -> WqT [I, O] codes + per-in-feature scales.  `ws` holds the partial column
// maxima and the reciprocal scales: quant_cols_ws_bytes(O, I) bytes.
size_t quant_cols_ws_bytes(int64_t O, int64_t I);
hipError_t launch_quant_cols(const void *W, int O, int I, int B, bool is_f32, uint32_t k0, uint32_t k1,
                             float qmax, bool packed, bool mant, int8_t *WqT, float *sW, float *coeffT, void *ws,
                             hipStream_t st);

// The same scratch as a file-scope device array inside the library (k_quant_cols.hip), for callers that
// cannot allocate: room for the column maxima of a weight with up to kQuantColsStaticMaxI in-features
// (256 KiB per GPU).  Returns the array's address on the current device (asked for once per device).
constexpr int kQuantColsStaticMaxI = 65536;
hipError_t quant_cols_static_scratch(void **ptr);

// Shape of a workgroup of K1T's two passes, as for K3: B lanes side by side (runs of 256 B of a row
// of bf16) times 256/B row blocks, whose codes are neighbours in a row of the transposed output
// (runs of 256 bytes, 128 packed).
inline int cols_grid_x(int I, int B) { return (I + 127) / 128; }
inline int cols_grid_y(int O, int B) { return (O + 255) / 256; }       // 256/B row blocks of B rows

// K1T split in its two passes, for callers that run pass 1 elsewhere (the fused front launches):
// pass 2 alone, reading the column maxima pass 1 left in `ws`.
hipError_t launch_quant_cols_pass2(const void *W, int O, int I, int B, bool is_f32, uint32_t k0, uint32_t k1,
                                   float qmax, bool packed, bool mant, int8_t *WqT, float *sW, float *coeffT,
                                   const void *ws, hipStream_t st);
// The weights that one workgroup per strip of columns quantises completely, both passes, inside the
// one-launch front (launch_front_one below): at most 256 row blocks (O / B; 64 groups of four lanes
// take one each per round, so four rounds a pass) and small enough for the second pass to find
// them in the cache.  Measured: a gain up to these sizes, none at 13-20 MB, a loss beyond.
constexpr int kColsFullMaxRowBlocks = 256;
constexpr int64_t kColsFullMaxBytes = 8 << 20;
bool cols_full_ok(int O, int I, int B, bool is_f32);

// Geometry of a convolution over channels-last tensors.  N = Nb * Ho * Wo rows of the column matrix.
struct ConvShape {
    int Nb, H, W, C, kh, kw, sh, sw, ph, pw, dh, dw, Ho, Wo;
    int64_t N;
};

// The independent transforms of one backward pass in two launches (k_front.hip).  A job with a
// null tensor is empty.
struct FrontRows {   // K1 on G, 256-thread variant
    const void *G;
    int64_t N;
    int O, T;
    uint32_t k0, k1;
    float qmax;
    int8_t *Gq;
    float *sG;
    int blocks;
};
struct FrontHla {    // K3 on one tensor
    const void *T;
    int64_t N;
    int D, r;
    uint16_t *out;
    int gx, gy;      // column strips of 128, groups of 256/B token blocks
    int grp, nb;     // hla_job_map's grouping and the workgroups it needs (>= gx * gy)
};
// Shape of a K3 workgroup: B lanes side by side (each CPL = 128/B columns: 256 B of a row of bf16
// whatever B) times 256/B token blocks, so that both the reads (runs of 256 B) and the writes
// (r coefficients of 256/B consecutive token blocks: 512 r/B bytes of an output row) come in long
// runs.  Measured at B = 16 on cold inputs against 64 lanes x 4 token blocks (1 KB reads, 8 r byte
// writes), us: X of 65536 x 576: 54.8 -> 25.1, G of 4096 x 11008: 41.7 -> 34.2, G of 12608 x 3072:
// 36.5 -> 27.5.  (16 lanes at B = 64 would read runs of 64 B: the whole pass 424 -> 451 us.)
constexpr int hla_lanes(int B) { return B; }
constexpr int hla_blocks(int B) { return 256 / B; }
inline int hla_grid_x(int D, int B) { return (D + 127) / 128; }      // B lanes x 128/B columns = 128 columns
inline int hla_grid_y(int64_t N, int B) { return static_cast<int>((N / B + hla_blocks(B) - 1) / hla_blocks(B)); }
// Order of the workgroups of a K3 job.  A workgroup writes 512 r/B bytes of each of its output rows
// and the workgroup of the next `by` the bytes after them; workgroups go round-robin to the eight
// XCDs (index mod 8), each with its own L2.  Where that is less than a 128-byte line, hla_job_map
// (hla_body.hpp) keeps the `grp` consecutive `by` that complete a line on one XCD, back to back, so
// that their pieces meet in that L2 and leave it as whole lines.
inline int hla_job_grp(int B, int r)
{
    const int bytes = 512 * r / B;
    return bytes >= 128 ? 1 : (bytes >= 64 ? 2 : (bytes >= 32 ? 4 : 8));
}
inline int hla_job_blocks(int gx, int gy, int grp)
{
    const int units = gx * ((gy + grp - 1) / grp);
    return 8 * grp * ((units + 7) / 8);
}
// K1(G) and K3(G) of one launch sharing ONE read of G from memory: rows of G go through in groups of
// 128; the workgroups of a group -- its K1 rows, then its K3 strips of 256 columns -- sit next to one
// another in the index sequence of ONE XCD (index mod 8), so that whichever of the two readers of a row
// comes second finds it in that XCD's L2.  `pair` consecutive groups (the ones whose K3 output pieces
// complete a 128-byte line) go to the same XCD back to back.  on == 0: the jobs keep their own ranges.
struct FrontShare {
    int on;
    int nk1;      // K1 workgroups per group of 128 rows
    int gx;       // K3 workgroups per group (strips of 256 columns)
    int pair;     // groups per unit handed to an XCD
    int units;    // units in all
    int blocks;   // workgroups of the two jobs together: 8 * ceil(units / 8) * pair * (nk1 + gx)
};
// The two jobs of the first launch in turns along the index sequence: `gran * q` workgroups of the row
// quantiser, then `gran` of the projection, `cyc` times over, then what is left of either.  The quantiser is
// bound by its arithmetic and the projection by memory: side by side on a compute unit they take less than
// one after the other.  gran == 0: each job keeps its own range of indices.
struct FrontMix {
    int gran, q, cyc;
};
struct FrontConv {   // on: the K3(X) job of front A reads the column matrix of an image (jx.T = the image)
    ConvShape g;
    int on;
};
struct FrontFill {   // n words at p := 0
    uint32_t *p;
    int n;
};
struct FrontAbsmax { // pass 1 of K1T
    const void *W;
    int O, I;
    uint32_t *amax;
    int gx, gy;
};
struct FrontHlaQ {   // K3 + int8 quantisation of one tensor: pass 1 (amax) and pass 2 (codes) read the same fields
    const void *T;
    int64_t N;
    int D, r;
    uint32_t *amax;
    uint32_t k0, k1;
    int8_t *TqT;
    float *sT;
    int gx, gy;
};
struct FrontColsQ {  // pass 2 of K1T
    const void *W;
    int O, I;
    const uint32_t *amax;
    uint32_t k0, k1;
    float qmax;
    int8_t *WqT;
    float *sW;
    int gx, gy;
};
FrontHlaQ front_hlaq(const void *T, int64_t N, int D, int B, int r, uint32_t *amax, uint32_t k0, uint32_t k1, int8_t *TqT,
                     float *sT);
FrontColsQ front_colsq(const void *W, int O, int I, int B, const uint32_t *amax, uint32_t k0, uint32_t k1, float qmax,
                       int8_t *WqT, float *sW);
// The integer g_w list in three launches: (K1(G) | zeroing) through launch_front with empty K3 jobs,
// then every pass 1 (maxima of projected G, projected X, transformed W), then every pass 2.  `jr`, if it is
// not empty, is K1(G) riding in the second launch instead, its workgroups in turns with the passes 1.
hipError_t launch_front_q(const FrontHlaQ &jg, const FrontHlaQ &jx, const FrontAbsmax &jw, const FrontColsQ &jq,
                          const FrontRows &jr, int B, int basis, bool is_f32, bool packed, hipStream_t st);
bool front_fusable(int O, int B);
FrontRows front_rows(const void *G, int64_t N, int O, int B, uint32_t k0, uint32_t k1, float qmax, int8_t *Gq, float *sG);
FrontHla front_hla(const void *T, int64_t N, int D, int B, int r, uint16_t *out);
FrontAbsmax front_absmax(const void *W, int O, int I, int B, uint32_t *amax);
// all of K1T for a weight that passes cols_full_ok: one workgroup per strip of columns (gy carries the
// strip's width as a shift)
FrontColsQ front_cols_full(const void *W, int O, int I, int B, uint32_t k0, uint32_t k1, float qmax, int8_t *WqT, float *sW);
// K1(G) | K3(X) | K3(G) | all of K1T in ONE launch (jq from front_cols_full, or without a weight):
// nothing has to be zeroed beforehand and no launch for pass 2 follows.
hipError_t launch_front_one(const FrontRows &jr, const FrontHla &jx, const FrontHla &jg, const FrontColsQ &jq,
                            const ConvShape *conv, int B, int basis, bool is_f32, bool packed, hipStream_t st);
// conv: NULL, or the geometry whose column matrix jx.T (an image) stands for; needs hla_conv_ok.
hipError_t launch_front(const FrontRows &jr, const FrontHla &jx, const FrontFill &jf, const FrontHla &jg,
                        const FrontAbsmax &jw, const ConvShape *conv, int B, int basis, bool is_f32, bool packed,
                        hipStream_t st);
// whether launch_front lets K1 (jr) and its first K3 job (jx) share the read of their tensor; switch for A/B
FrontShare front_share(const FrontRows &jr, const FrontHla &jx, int B, bool is_f32);
void front_share_enable(bool on);
void front_mix_enable(bool on);
bool front_mix_enabled();

// K3: token-axis Hadamard low-rank projection, T [N, D] -> ThatT [D, N/B*r] bf16.
// basis: which r rows of the order-B matrix are kept, 0 = rows 0..r-1, 1 = the r of lowest sequency.
hipError_t launch_hla(const void *T, int64_t N, int D, int B, int r, int basis, bool is_f32, uint16_t *ThatT,
                      float *coeffT, hipStream_t st);

// K3q: token-axis projection followed by int8 quantisation with one scale per feature (stages
// 1-2 / 3-4 of the g_w list): T [N, D] -> TqT [D, N/B*r] int8 + sT [D].  `ws` holds D words of
// column maxima: hla_quant_ws_bytes(D) bytes.  Needs r % 4 == 0.
size_t hla_quant_ws_bytes(int64_t D);
// p4: codes in [-7, 7] stored two to a byte (TqT [D, N/B*r/2] bytes; needs r % 8 == 0; seeded rounding only)
hipError_t launch_hla_quant(const void *T, int64_t N, int D, int B, int r, int basis, bool is_f32, uint32_t k0,
                            uint32_t k1, bool mant, int8_t *TqT, float *sT, float *coeffT, void *ws, hipStream_t st,
                            bool p4 = false);
// 4-bit codes two to a byte -> one int8 each; bytes_in a multiple of 16, both pointers 16-byte aligned
hipError_t launch_unpack_nibbles(const void *in, int8_t *out, int64_t bytes_in, hipStream_t st);

// K2 / K4: C = alpha * sA (x) sB * (A . Bm^T).  kind 0: int8 operands, int32 accumulate;
// kind 1: bf16 operands, fp32 accumulate.  K in elements.
struct GemmArgs {
    const void *A;
    const void *Bm;
    int M, N, K;
    const float *sA;
    const float *sB;
    float alpha;
    void *C;          // bf16 or fp32 [M, N], may be null
    bool c_is_f32;
    int32_t *acc;     // raw int32 accumulators (int8 kind only), may be null
    void *ws;         // device scratch for split-K partial sums, may be null (then k is never split)
    size_t ws_bytes;
};
hipError_t launch_gemm_nt(int kind, const GemmArgs &a, hipStream_t st);
hipError_t launch_splitk_reduce(int kind, const GemmArgs &a, int splits, hipStream_t st);
// The same reduction as a job description, for a later launch of the caller's that carries it
// beside its own work (the fold of a convolution): `blocks` workgroups of 256 threads, 0 = none.
struct SplitReduce {
    const int32_t *partial;
    int splits, M, N;
    const float *sA, *sB;
    float alpha;
    void *C;
    int kind, c_is_f32;
    int blocks;
};
SplitReduce splitk_reduce_job_of(int kind, const GemmArgs &a, int splits);
// K2 | K4 in one launch (k_gemm_pair.hip): product `a` of kind 2 and product `b` of kind 1, both
// with a scaled output of the same dtype.  Only b's k may be split (b.ws).  gemm_pair_available
// says whether the combination is built; the results are those of two launch_gemm_nt calls up to
// the summation order of b's k splits.
bool gemm_pair_available(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b);
// defer: if not null and b's k is split, the reduction is not launched but described there (blocks > 0).
hipError_t launch_gemm_pair(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b, hipStream_t st,
                            SplitReduce *defer = nullptr);
// The products as ONE persistent launch (k_gemm_stream.hip): a workgroup per compute unit walks a
// fixed list of 256 x 256 tiles of `a`, then of `b` (NULL: one product only), loading across tile
// boundaries.  Same bits as launch_gemm_nt without a k split.  gemm_stream_wanted: the shapes allow it
// (bf16 output, whole k steps, at least four tiles per compute unit in all) and it has not been
// switched off; callers ask it after their plan has chosen 256-tiles and no k split.
bool gemm_stream_wanted(int kindA, const GemmArgs &a, int kindB, const GemmArgs *b);
hipError_t launch_gemm_stream(int kindA, const GemmArgs &a, int kindB, const GemmArgs *b, hipStream_t st);
void gemm_stream_enable(bool on);
void gemm_dl_enable(bool on);   // operands of 256-tiles straight into LDS where the shape allows (default on)
void gemm_tail_enable(bool on);   // 192-row tiles for the last rows of a product whose last round would be partly empty (default on)
void gemm_plan_force(int tile, int splits);   // measurement overrides of the plans, see gemm_plan.hpp
// What launch_gemm_pair would do with these shapes and this much split-k scratch, without doing it:
// plan[0], plan[1] = tile edge (256 or 128) of a's and b's product, plan[2] = k splits of b,
// plan[3] = 1 if b's tiles are dispatched first, plan[4] = 1 if the persistent form takes the launch.
void gemm_pair_describe(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b, size_t ws_bytes, int plan[5]);
// split-k scratch (b.ws) that the pair's plan would use if it may have up to `cap` bytes; only the
// shapes and kinds of a and b are read
size_t gemm_pair_ws_bytes(int kindA, const GemmArgs &a, int kindB, const GemmArgs &b, size_t cap);
// Scratch that lets launch_gemm_nt split k whenever that is the faster plan for this shape
// (few output tiles, long reduction); 0 if the plan does not split.
size_t gemm_ws_bytes(int kind, int M, int N, int K);

// Convolution glue (k_conv.hip), channels-last tensors.
// x [Nb, H, W, C] -> cols [N, kh*kw*C], columns ordered (ky, kx, c), zero padding
hipError_t launch_im2col(const void *X, const ConvShape &g, bool is_f32, void *cols, hipStream_t st);
// cols [N, kh*kw*C] -> dx [Nb, H, W, C]: each pixel sums the entries copied from it (fp32, fixed order)
// red: NULL, or a split-K reduction (independent of the fold) that the first red->blocks workgroups run
hipError_t launch_col2im(const void *cols, const ConvShape &g, bool is_f32, void *dx, hipStream_t st,
                         const SplitReduce *red = nullptr);

// K3 / K3q on the column matrix of X [Nb, H, W, C] without storing it: same outputs as launch_hla /
// launch_hla_quant on launch_im2col's result, D = kh*kw*C.  Needs hla_conv_ok (C a multiple of the
// 128 / B features a lane owns).
bool hla_conv_ok(const ConvShape &g, int B);
hipError_t launch_hla_conv(const void *X, const ConvShape &g, int B, int r, int basis, bool is_f32, uint16_t *ThatT,
                           float *coeffT, hipStream_t st);
hipError_t launch_hla_quant_conv(const void *X, const ConvShape &g, int B, int r, int basis, bool is_f32, uint32_t k0,
                                 uint32_t k1, bool mant, int8_t *TqT, float *sT, float *coeffT, void *ws, hipStream_t st);

// Diagnostic: `blocks` workgroups of 4 wavefronts each run `iters` x 8 independent 32x32 MFMAs
// (kind 0: i8, K = 32; kind 1: bf16, K = 16) from registers.
hipError_t launch_mfma_probe(int kind, int blocks, int iters, float *sink, hipStream_t st);

}  // namespace hlq
