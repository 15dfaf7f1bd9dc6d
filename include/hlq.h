/*
 * hlq.h -- C ABI of the MI355X (gfx950) HLQ backward-pass library.
 *
 * HLQ = Hadamard Low-rank Quantization (arXiv 2406.15102): the backward pass of a linear
 * (or im2col'd convolution) layer y = x w^T (Sec. 3.1, Eq. 1) computed as
 *
 *   dX = Q(G H_O) . Q(H_O^T W)          activation gradient, Sec. 5.1 and the six g_x stages of Sec. 6.1
 *   dW = (G^T H_L^T)(H_L X), r of B      weight gradient, Sec. 4 / 5.1 and stages 1, 3, 5 of the six
 *        bases kept per token block      g_w stages of Sec. 6.1 (operands kept in bf16, not int8)
 *
 * with the block-diagonal Walsh-Hadamard transform of Sec. 3.2 and the 4-bit stochastic
 * quantiser of Sec. 5.1 / 6.1.
 *
 * Notation (paper -> here): tokens B*L -> N; I -> d_in; O -> d_out; Hadamard order n -> B;
 * kept bases r -> r.  G = g_y as [N, d_out], X = x as [N, d_in], W = w as [d_out, d_in].
 *
 * General conventions
 *   - Every tensor argument is a DEVICE pointer to a dense row-major array owned by the caller,
 *     16-byte aligned; the library reads inputs, writes outputs, keeps no reference after return.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; no call synchronises the device.  Except where noted, no call allocates.
 *   - `dtype` selects the element type of G, X, W and of dX, dW: HLQ_BF16 or HLQ_F32.
 *     Arithmetic is fp32 (transforms, scales), int8 x int8 -> int32 (dX product) and
 *     bf16 x bf16 -> fp32 (dW product) whatever the dtype.
 *   - Every function returns an hlq_status.  On any status other than HLQ_OK nothing has been
 *     enqueued and no output byte is written (HLQ_ERR_LAUNCH excepted: an earlier kernel of the
 *     same call may already be queued).
 *   - Same inputs and seed give bit-identical outputs on every call.
 *
 * Shape rules (violations give the listed status)
 *   B in {16, 32, 64}                               HLQ_ERR_BLOCK
 *   r a power of two, 1 <= r <= B                   HLQ_ERR_RANK
 *   N > 0, N % B == 0; d_out > 0, d_out % B == 0, d_out <= 65536;
 *   d_in > 0, d_in % 8 == 0; (N / B * r) % 8 == 0;
 *   N * d_out / 4 < 2^32 and d_in * d_out / 4 < 2^32 (random-stream counters);
 *   N / B <= 262140 and ceil(D / 128) * ceil(N / (4 B)) < 2^30 for D = d_in and D = d_out
 *   (workgroups of one launch of the token-axis transform)                        HLQ_ERR_SHAPE
 */
#ifndef HLQ_H_
#define HLQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hlq_status {
    HLQ_OK = 0,
    HLQ_ERR_NULL = 1,      /* a required pointer is NULL */
    HLQ_ERR_SHAPE = 2,     /* a size breaks the shape rules above */
    HLQ_ERR_BLOCK = 3,     /* B not in {16, 32, 64} */
    HLQ_ERR_RANK = 4,      /* r not a power of two in [1, B] */
    HLQ_ERR_DTYPE = 5,     /* dtype not HLQ_BF16 / HLQ_F32 */
    HLQ_ERR_WORKSPACE = 6, /* workspace too small, misaligned, or could not be allocated */
    HLQ_ERR_LAUNCH = 7     /* the HIP runtime refused a launch */
} hlq_status;

typedef enum hlq_dtype { HLQ_BF16 = 0, HLQ_F32 = 1 } hlq_dtype;

/* Human-readable name of a status (static string, never NULL). */
const char *hlq_status_str(int status);

/* Library version, major*10000 + minor*100 + patch. */
int hlq_version(void);

/*
 * Bytes of device scratch hlq_linear_backward_ex needs for this problem (quantised operands,
 * scales, partial column maxima, HLA-compressed operands).  Returns 0 if the shape is invalid.
 * `x_is_compressed` != 0 sizes it for a call that passes XhatT instead of X.
 */
size_t hlq_workspace_bytes(int64_t N, int64_t d_in, int64_t d_out, int B, int r, int x_is_compressed);

/*
 * Process-wide switches, for measurements (every setting computes the same results; see PLAN_SPLITS for
 * the one qualification).
 *   HLQ_OPT_PERSISTENT_PRODUCTS  1: layers whose matrix products (Sec. 6.1, g_x stages 5-6 and g_w
 *       stage 5) come to at least four 256 x 256 tiles per compute unit run them as one persistent
 *       launch, a workgroup per compute unit walking a fixed list of tiles and loading across tile
 *       boundaries (operands staged through registers);  0 (default): always one workgroup per tile.
 *   HLQ_OPT_SHARED_G_READ  1: for a large G, the workgroups that quantise a group of 128 rows of
 *       G (g_x stages 1-2) and those that project the same rows along the tokens (g_w stage 3) are
 *       dispatched next to one another on one XCD, so that the second reader finds the rows in that
 *       XCD's L2 and G comes from memory once (measured at N = 4096, d_out = 11008: 98.5 MB fetched
 *       instead of 180.6 MB, 51.5 instead of 53.0 us -- the launch is not bound by those bytes);
 *       0 (default): each stage's workgroups keep their own index range.
 *   HLQ_OPT_DIRECT_TO_LDS  1 (default): 256 x 256 tiles of the matrix products whose operand rows are
 *       whole 128-byte steps (at least four per workgroup) load their operands from global memory
 *       straight into LDS;  0: every tile stages them through registers.
 *   HLQ_OPT_TAIL_TILES  1 (default): a product on 256 x 256 tiles that loads straight into LDS and would
 *       leave most compute units idle in its last round hands its last rows to tiles of 192 x 256, which
 *       shortens that round by a quarter (the g_w product when it closes the launch of both products, or a
 *       product launched alone; not the packed codes);  0: 256 x 256 tiles throughout.
 *   HLQ_OPT_FRONT_INTERLEAVE  1 (default): the row quantiser of G shares a launch with all the
 *       memory-bound transforms that do not wait for anything -- both token-axis projections, or, on the
 *       integer g_w list, the passes that take the maxima -- and the workgroups of the two kinds take
 *       turns along the index sequence (the quantiser is bound by arithmetic: side by side they take
 *       less);  0: the former composition -- the quantiser's workgroups first, then one projection, the
 *       other in the second launch (integer g_w list: the quantiser with the zeroing, before the passes).
 *   HLQ_OPT_PLAN_TILE  0 (default): a cost model picks 128 x 128 or 256 x 256 tiles for each matrix product;
 *       128 or 256: every product takes that tile.
 *   HLQ_OPT_PLAN_SPLITS  0 (default): the model picks the k split of a product with few output tiles (of
 *       the g_w product when the two share a launch);  1..16: that split, cut down to the steps of the
 *       reduction and to the split-k scratch at hand.  The workspace sizes are computed under the same
 *       setting, so set it before asking for them.  A different split sums the bf16 product in a
 *       different order: dW then agrees to rounding, not bit for bit; everything else stays bit-equal.
 * Unknown option or value: HLQ_ERR_SHAPE.  Not synchronised with calls running on other host threads.
 */
#define HLQ_OPT_PERSISTENT_PRODUCTS 1
#define HLQ_OPT_SHARED_G_READ 2
#define HLQ_OPT_DIRECT_TO_LDS 3
#define HLQ_OPT_PLAN_TILE 4
#define HLQ_OPT_PLAN_SPLITS 5
#define HLQ_OPT_TAIL_TILES 6
#define HLQ_OPT_FRONT_INTERLEAVE 7
int hlq_set_option(int option, int value);

/*
 * Registers caller-owned device memory as the scratch of every call on the CURRENT device that is
 * given no workspace of its own (hlq_linear_backward, and the entry points below when their
 * `workspace` is NULL): the layer of Sec. 3.1, Eq. 1 then runs through the plain signature without
 * the library ever allocating, freeing or synchronising.
 *   dev_ptr  256-byte aligned device memory that stays valid until it is replaced or withdrawn;
 *            NULL (bytes ignored) withdraws the registration and returns to the library-owned scratch.
 *   bytes    its size; size it with hlq_workspace_bytes / hlq_workspace_bytes_mode /
 *            hlq_conv_workspace_bytes for the largest problem that will be run.
 * HLQ_ERR_WORKSPACE for a misaligned pointer or bytes == 0 with a non-NULL pointer (the previous
 * registration stays).  The memory is not touched by this call.  Host-side only: no GPU work.
 */
int hlq_set_workspace(void *dev_ptr, size_t bytes);

/*
 * The whole backward pass of one layer for bf16 tensors (both stage lists of Sec. 6.1):
 *   dX [N, d_in]     = dequant( Q4(G H) . Q4(H^T W) )        stages 1-6 of the g_x list
 *   dW [d_out, d_in] = (1/B) . HLA_r(G)^T . HLA_r(X)          stages 1, 3, 5 of the g_w list
 * `seed` selects the stochastic-rounding stream (same seed -> same bits).
 * Scratch memory: the workspace registered with hlq_set_workspace for the current device, if any --
 * the call then allocates nothing, frees nothing and never synchronises, and returns
 * HLQ_ERR_WORKSPACE (nothing enqueued) when hlq_workspace_bytes(...) exceeds what was registered.
 * With nothing registered the library owns the scratch: allocated with hipMalloc on the first call
 * on a device and again only when a later call needs more (such a call synchronises the device and
 * frees the old buffer: outside any hot path, never under stream capture).
 * Calls that share a workspace -- registered or library-owned -- must not overlap on one device,
 * whether from two streams or two host threads.
 */
int hlq_linear_backward(const void *G, const void *X, const void *W, int64_t N, int64_t d_in,
                        int64_t d_out, int B, int r, uint64_t seed, void *dX, void *dW, void *stream);

/*
 * As above with every option spelled out.
 *   X      [N, d_in] or NULL;  XhatT [d_in, N/B*r] bf16 or NULL: exactly one of the two when dW is
 *          wanted.  XhatT is what hlq_compress_act stored at forward time (ACBP, Sec. 6.1).
 *   dX, dW either may be NULL to skip that half (X/XhatT may then be NULL when dW is NULL, and
 *          W may be NULL when dX is NULL).
 *   workspace  device memory of at least hlq_workspace_bytes(...) bytes, 256-byte aligned, or
 *          NULL to use the registered or library-owned workspace described above.
 */
int hlq_linear_backward_ex(const void *G, const void *X, const void *XhatT, const void *W, int64_t N,
                           int64_t d_in, int64_t d_out, int B, int r, uint64_t seed, int dtype,
                           void *dX, void *dW, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Activation compression for backward propagation (ACBP, Sec. 6.1): stage 1 of the g_w list
 * applied to X at forward time.  For token block b and feature j,
 *   XhatT[j, b*r + k] = bf16( sum_n H[k][n] X[b*B + n, j] ),  k < r,
 * H the +-1 natural-order Walsh-Hadamard matrix of order B (Sec. 3.2), i.e. the first r of every
 * B coefficients, stored [d_in, N/B*r] bf16 with the compressed token axis contiguous.
 */
int hlq_compress_act(const void *X, int64_t N, int64_t d_in, int B, int r, int dtype, void *XhatT,
                     void *stream);

/* ---- stage entry points (the steps above one by one; also what the parity tests probe) ---- */

/* `bits` of hlq_quantize_g / hlq_quantize_w */
#define HLQ_BITS_4 4            /* codes in [-7, 7] (the method's setting), one int8 each */
#define HLQ_BITS_8 8            /* codes in [-127, 127] (the int8 warm-up phase of Sec. 7), one int8 each */
#define HLQ_BITS_4_PACKED 0x104 /* codes in [-7, 7], two to a byte: code 2b in the low nibble of byte b,
                                   code 2b+1 in the high nibble, two's complement; rows of d_out/2 bytes;
                                   needs d_out % 32 == 0.  The operand format of hlq_int4_gemm_nt. */

#define HLQ_BITS_ROUND_MANTISSA 0x200 /* OR into any of the above: round by the low 11 bits of each value's own
                                        fp32 pattern, u = (bits + 0.5) / 2048 -- the pseudo-stochastic quantiser
                                        the paper describes (Sec. 6.1) -- instead of the seeded stream (seed is
                                        then ignored).  Only as random as those bits: on coefficients of bf16
                                        inputs it mostly rounds down. */

/*
 * Stages 1-2 of the g_x list: block Hadamard transform of every row of G along d_out, then
 * stochastic quantisation with one absmax scale per row.
 *   bits  one of HLQ_BITS_*; anything else: HLQ_ERR_DTYPE.  The codes are the same for HLQ_BITS_4
 *         and HLQ_BITS_4_PACKED; only their storage differs.
 *   Gq [N, d_out] int8 (packed: [N, d_out/2] bytes);  sG [N] fp32, sG[n] = max|coef| / qmax.
 *   coeff: NULL, or [N, d_out] fp32 receiving the transformed values (unnormalised H).
 */
int hlq_quantize_g(const void *G, int64_t N, int64_t d_out, int B, uint64_t seed, int dtype, int bits,
                   int8_t *Gq, float *sG, float *coeff, void *stream);

/*
 * Stages 3-4 of the g_x list: H^T W (blocks of B consecutive rows of W are mixed), quantised
 * with one scale per in-feature and stored transposed, reduction axis contiguous:
 *   WqT [d_in, d_out] int8 (packed: [d_in, d_out/2] bytes);  sW [d_in] fp32;  coeffT: NULL or
 *   [d_in, d_out] fp32.  bits: as for hlq_quantize_g.
 *   workspace: >= hlq_quantize_w_workspace_bytes(d_out, d_in) bytes of device scratch (256-aligned).
 */
size_t hlq_quantize_w_workspace_bytes(int64_t d_out, int64_t d_in);
int hlq_quantize_w(const void *W, int64_t d_out, int64_t d_in, int B, uint64_t seed, int dtype, int bits,
                   int8_t *WqT, float *sW, float *coeffT, void *workspace, size_t workspace_bytes,
                   void *stream);

/*
 * hlq_quantize_w for callers that cannot allocate device memory and have no scratch to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results (WqT, sW bit for bit) minus coeffT and the workspace: the column maxima
 * live in a 256 KiB array inside the library's code object (one copy per GPU, kept until the
 * process ends).  Nothing is allocated or freed, by this call or by anything it calls.
 *   d_in <= 65536 (the array's size); beyond that HLQ_ERR_WORKSPACE, nothing enqueued.
 * Every call on a GPU uses that GPU's one array (zeroed by a fill kernel at the start of each call):
 * calls that overlap on one GPU -- two streams, two threads -- race; keep them on one stream.
 */
int hlq_quantize_w_static(const void *W, int64_t d_out, int64_t d_in, int B, uint64_t seed, int dtype, int bits,
                          int8_t *WqT, float *sW, void *stream);

/*
 * Stages 5-6 of the g_x list: C[m, n] = alpha * sA[m] * sB[n] * sum_k A[m,k] * Bm[n,k], the sum
 * exact in int32 (int8 MFMA).  A [M, K] int8, Bm [Nn, K] int8 with |value| <= 127, K % 16 == 0,
 * K <= 131072 (so that 127 * 127 * K fits int32), Nn % 4 == 0.
 *   out_dtype HLQ_BF16 / HLQ_F32 selects the type of C [M, Nn]; C may be NULL.
 *   acc: NULL or [M, Nn] int32 receiving the raw accumulators.  sA, sB may be NULL (= all ones).
 *   workspace: NULL, or device scratch (16-byte aligned) of hlq_gemm_workspace_bytes(0, M, Nn, K)
 *   bytes or more.  With it, shapes with few output tiles and a long reduction are computed as
 *   several partial products over ranges of k, summed in a fixed order (integers: exactly) by a
 *   second kernel; without it, or when it is too small, k is never split.  Same result either way
 *   for the int8 product; for the bf16 product the fp32 summation order differs.
 */
size_t hlq_gemm_workspace_bytes(int kind /* 0 int8, 1 bf16, 2 packed 4-bit */, int64_t M, int64_t Nn, int64_t K);
int hlq_int8_gemm_nt(const int8_t *A, const int8_t *Bm, int64_t M, int64_t Nn, int64_t K,
                     const float *sA, const float *sB, float alpha, int out_dtype, void *C,
                     int32_t *acc, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same product on 4-bit codes stored two to a byte (the paper's int4 operands, Sec. 6.1):
 * byte b of a row holds code 2b in its low nibble and code 2b+1 in its high nibble, two's
 * complement, |code| <= 7.  Half the bytes of the int8 layout in HBM, L2 and LDS; the nibbles are
 * widened to int8 MFMA operands in registers.  C and acc equal those of hlq_int8_gemm_nt on the
 * same codes bit for bit.
 *   A [M, K/2 bytes], Bm [Nn, K/2 bytes]; K % 32 == 0, K <= 131072, Nn % 4 == 0.
 *   Other arguments as for hlq_int8_gemm_nt (workspace: kind 2).
 */
int hlq_int4_gemm_nt(const void *A, const void *Bm, int64_t M, int64_t Nn, int64_t K, const float *sA,
                     const float *sB, float alpha, int out_dtype, void *C, int32_t *acc, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * Stages 1 and 3 of the g_w list for any [N, D] tensor T (G or X): the projection described at
 * hlq_compress_act.  ThatT [D, N/B*r] bf16;  coeffT: NULL or [D, N/B*r] fp32 receiving the
 * coefficients before rounding to bf16.
 */
int hlq_hla_project(const void *T, int64_t N, int64_t D, int B, int r, int dtype, void *ThatT,
                    float *coeffT, void *stream);

/*
 * Which r of the B coefficients "the first r" are (Sec. 6.1 follows the base selection of LBP-WHT,
 * which the paper does not spell out; Sec. 4 speaks of the low-frequency components of g_w).
 *   HLQ_BASIS_NATURAL   rows 0..r-1 of the matrix as Eq. 2 builds it -- what every entry point
 *                       without a basis argument uses;
 *   HLQ_BASIS_SEQUENCY  the r rows with the fewest sign changes, in that order (Walsh ordering):
 *                       a true low-pass, for r = B/2^m the averages over runs of B/r tokens.
 * Same arguments as hlq_hla_project otherwise; any other basis: HLQ_ERR_RANK.  For the forward-time
 * stores call these with T = X (and tensor = 2 for the integer one).
 */
#define HLQ_BASIS_NATURAL 0
#define HLQ_BASIS_SEQUENCY 1
#define HLQ_BASIS_ROUND_MANTISSA 0x200 /* hlq_hla_quantize_basis only, OR into the basis: rounding as
                                          HLQ_BITS_ROUND_MANTISSA */
int hlq_hla_project_basis(const void *T, int64_t N, int64_t D, int B, int r, int basis, int dtype, void *ThatT,
                          float *coeffT, void *stream);

/*
 * Stage 5 of the g_w list: C[m, n] = alpha * sum_k A[m,k] * Bm[n,k], bf16 inputs, fp32
 * accumulation (bf16 MFMA).  A [M, K], Bm [Nn, K] bf16, K % 8 == 0, Nn % 4 == 0; C [M, Nn] of
 * out_dtype.  workspace: as for hlq_int8_gemm_nt (kind 1).
 */
int hlq_bf16_gemm_nt(const void *A, const void *Bm, int64_t M, int64_t Nn, int64_t K, float alpha,
                     int out_dtype, void *C, void *workspace, size_t workspace_bytes, void *stream);

/* ---- the method's two options: 8-bit g_x codes, and the g_w list in integers ------------------- */

/* flags of hlq_linear_backward_mode / hlq_workspace_bytes_mode */
#define HLQ_FLAG_GX_8BIT 1 /* g_x codes in [-127, 127]: the int8 warm-up phase of Sec. 7 */
#define HLQ_FLAG_GW_INT8 2 /* g_w list in full (Sec. 6.1): projected X and G quantised to int8
                              (stages 2, 4), integer product (5), dequantisation (6) */
#define HLQ_FLAG_GW_SEQUENCY 8 /* g_w list keeps the r lowest-sequency coefficients (HLQ_BASIS_SEQUENCY); a
                                 forward-time store handed over as Xc must have been made the same way */
#define HLQ_FLAG_ROUND_MANTISSA 16 /* every quantiser of both lists rounds by the values' low 11 mantissa bits
                                     (HLQ_BITS_ROUND_MANTISSA); one launch per stage */
#define HLQ_FLAG_SEPARATE_PRODUCTS 32 /* one launch per matrix product.  By default the two products of the
                                        default lists share a launch (they are independent, and neither fills
                                        the chip for most layers); dX is the same bit for bit either way, dW
                                        up to the summation order of its k splits. */
#define HLQ_FLAG_GX_UNPACKED 4 /* keep the 4-bit g_x codes one per int8 between the stages.  By default
                                  they are stored two to a byte whenever d_out % 32 == 0 (same codes, same
                                  dX bit for bit; half the traffic). */

/*
 * Stages 1-2 (T = X, tensor 2) or 3-4 (T = G, tensor 3) of the g_w list: the projection described
 * at hlq_compress_act followed by int8 stochastic quantisation (codes in [-127, 127]) with one
 * absmax scale per feature:
 *   TqT [D, N/B*r] int8;  sT [D] fp32;  coeffT: NULL or [D, N/B*r] fp32 (coefficients before
 *   quantisation).  Needs r % 4 == 0 (HLQ_ERR_RANK) and (N/B*r) % 16 == 0 (HLQ_ERR_SHAPE).
 *   tensor: 2 or 3, selects the random stream (HLQ_ERR_SHAPE otherwise).
 *   workspace: >= hlq_hla_quantize_workspace_bytes(D) bytes of device scratch (256-aligned).
 */
size_t hlq_hla_quantize_workspace_bytes(int64_t D);
int hlq_hla_quantize(const void *T, int64_t N, int64_t D, int B, int r, uint64_t seed, int tensor, int dtype,
                     int8_t *TqT, float *sT, float *coeffT, void *workspace, size_t workspace_bytes,
                     void *stream);
int hlq_hla_quantize_basis(const void *T, int64_t N, int64_t D, int B, int r, int basis, uint64_t seed, int tensor,
                           int dtype, int8_t *TqT, float *sT, float *coeffT, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * ACBP with integer storage (Sec. 6.1: "apply stages 1 and 2 during forward propagation and store
 * the intermediate feature map" in integers): hlq_hla_quantize on X with tensor 2.
 * XqT [d_in, N/B*r] int8, sX [d_in] fp32: a quarter (r = B/2) of X's bf16 footprint.
 */
int hlq_compress_act_int8(const void *X, int64_t N, int64_t d_in, int B, int r, uint64_t seed, int dtype,
                          int8_t *XqT, float *sX, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ACBP with the 4-bit store the paper names (Sec. 6.1: the compressed activation is kept as int4, an
 * eighth of an fp32 feature map before the r/B reduction): stage 2 of the g_w list with codes in
 * [-7, 7] -- same projection, same random stream (tensor 2) and counters, same per-feature absmax
 * as hlq_compress_act_int8, scale sX = absmax / 7 -- stored two to a byte in the layout of
 * HLQ_BITS_4_PACKED:  Xq4T [d_in, N/B*r/2] bytes, sX [d_in] fp32: an eighth (r = B/2) of X's bf16
 * footprint.  Needs r % 8 == 0 (HLQ_ERR_RANK) and (N/B*r) % 32 == 0 (HLQ_ERR_SHAPE); workspace as
 * for hlq_compress_act_int8.  The backward pass takes it as Xc with HLQ_FLAG_GW_INT8 | HLQ_FLAG_XC_INT4:
 * the codes are widened to int8 (a pass over the store, into the workspace) and multiplied with the
 * int8 codes of the projected gradient; dW = acc * sGhat[o] * sX[i] / B as in the int8 list.
 */
#define HLQ_FLAG_XC_INT4 64 /* Xc holds 4-bit codes two to a byte (hlq_compress_act_int4); needs HLQ_FLAG_GW_INT8 and Xc */
int hlq_compress_act_int4(const void *X, int64_t N, int64_t d_in, int B, int r, uint64_t seed, int dtype,
                          uint8_t *Xq4T, float *sX, void *workspace, size_t workspace_bytes, void *stream);

/*
 * hlq_linear_backward_ex with the options above.
 *   Xc, sXc   X compressed at forward time, or NULL: bf16 XhatT (sXc NULL) without
 *             HLQ_FLAG_GW_INT8; int8 XqT with its scales sXc [d_in] with it (4-bit Xq4T with
 *             HLQ_FLAG_XC_INT4 as well).  Exactly one of X and Xc when dW is wanted.
 *   flags     any combination of HLQ_FLAG_*; 0 = hlq_linear_backward_ex.
 *   workspace >= hlq_workspace_bytes_mode(...) bytes, 256-aligned, or NULL for the library-owned one.
 * HLQ_FLAG_GW_INT8 additionally needs r % 4 == 0 (HLQ_ERR_RANK), (N/B*r) % 16 == 0 and N/B*r <= 131072.
 */
size_t hlq_workspace_bytes_mode(int64_t N, int64_t d_in, int64_t d_out, int B, int r, int x_is_compressed,
                                int flags);
int hlq_linear_backward_mode(const void *G, const void *X, const void *Xc, const float *sXc, const void *W,
                             int64_t N, int64_t d_in, int64_t d_out, int B, int r, uint64_t seed, int dtype,
                             int flags, void *dX, void *dW, void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * The same with the weight operand quantised beforehand: the weight changes once per optimiser
 * step, its codes can serve every micro-batch in between (same seed => the codes the path itself
 * would compute, so the results are those of hlq_linear_backward_mode bit for bit).
 *   WqT, sW   as written by hlq_quantize_w(W, ..., seed, ..., bits = hlq_weight_code_bits(d_out, flags)):
 *             that helper returns the HLQ_BITS_* value (storage included) this path expects for
 *             the given flags.  Ignored (may be NULL) when dX is NULL.
 *   Other arguments, workspace and errors as for hlq_linear_backward_mode.
 */
int hlq_weight_code_bits(int64_t d_out, int flags);
int hlq_linear_backward_cached(const void *G, const void *X, const void *Xc, const float *sXc, const void *WqT,
                               const float *sW, int64_t N, int64_t d_in, int64_t d_out, int B, int r,
                               uint64_t seed, int dtype, int flags, void *dX, void *dW, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * Diagnostic, not part of the backward pass: `blocks` workgroups of four wavefronts each issue
 * iters * 8 independent MFMAs from registers (kind 0: int8 32x32x32 on random bytes, 65536 ops each;
 * kind 1: bf16 32x32x16, 32768 flops each; 2, 3, 4: fp8, fp6, fp4 32x32x64; 5: bf16 16x16x32, 16384
 * flops each; 6: int8 16x16x64, 32768 ops each; 7, 8: int8 32x32x32 on 4-bit codes times 16 -- what
 * the packed-code product feeds -- and on the codes as small integers; 9: int8 16x16x64 on the codes
 * times 16).  Timing it gives the MFMA
 * rate the chip sustains at its running clock for that shape and operand pattern, the practical
 * ceiling for the two matrix products of Sec. 6.1; kind outside 0..9: HLQ_ERR_SHAPE.
 * sink: one device float (never written in practice; keeps the loop alive).
 */
int hlq_mfma_probe(int kind, int blocks, int iters, float *sink, void *stream);

/*
 * Stages 5-6 of the g_x list and stage 5 (and 6) of the g_w list in ONE launch -- what the whole
 * path runs after its transforms.  The two products are independent and for most layers neither
 * fills the chip: tiles of one take the compute units the other leaves idle.
 *   Gq [N, d_out] / WqT [d_in, d_out] codes as hlq_quantize_g / _w store them for `gx_bits`
 *   (HLQ_BITS_4, HLQ_BITS_8 or HLQ_BITS_4_PACKED, no rounding bit), with sG [N], sW [d_in];
 *   GhatT [d_out, Kc] / XhatT [d_in, Kc]: bf16 projections (sGhat = sXhat = NULL), or int8 codes with
 *   their scales sGhat [d_out], sXhat [d_in] (the integer g_w list);
 *   dX [N, d_in] = Gq . WqT^T * sG (x) sW / B,  dW [d_out, d_in] = GhatT . XhatT^T (* scales) / B, of `dtype`.
 *   workspace: NULL, or >= hlq_backward_products_workspace_bytes(...) bytes of device scratch
 *   (16-byte aligned) that lets the g_w product split its reduction.
 * Shape rules of the two products (hlq_int8_gemm_nt / hlq_int4_gemm_nt / hlq_bf16_gemm_nt) apply.
 * dX equals the single product's bit for bit; dW up to the summation order of the k splits.
 */
size_t hlq_backward_products_workspace_bytes(int64_t N, int64_t d_in, int64_t d_out, int64_t Kc, int gx_bits, int gw_int8);
/*
 * How hlq_backward_products would lay the two products out for bf16 outputs, given `workspace_bytes` of
 * split-k scratch -- host arithmetic only, nothing is launched (the plan is a cost model fitted to
 * measurements; this entry point lets a test pin its choices):
 *   plan[0], plan[1]  tile edge (256 or 128) of the g_x and of the g_w product
 *   plan[2]           k splits of the g_w product
 *   plan[3]           1 if the g_w product's tiles are dispatched first
 *   plan[4]           1 if the persistent form takes the launch (needs a visible GPU: its grid is the
 *                     number of compute units; 0 without one)
 * Status codes as for hlq_backward_products_workspace_bytes's shape rules; plan NULL: HLQ_ERR_NULL.
 */
int hlq_backward_products_plan(int64_t N, int64_t d_in, int64_t d_out, int64_t Kc, int gx_bits, int gw_int8,
                               size_t workspace_bytes, int *plan);
int hlq_backward_products(const void *Gq, const float *sG, const void *WqT, const float *sW, int gx_bits,
                          const void *GhatT, const float *sGhat, const void *XhatT, const float *sXhat, int64_t N,
                          int64_t d_in, int64_t d_out, int64_t Kc, int B, int dtype, void *dX, void *dW, void *workspace,
                          size_t workspace_bytes, void *stream);

/* ---- convolution layers ------------------------------------------------------------------------ */

/*
 * Sec. 3.1: a convolution is optimised by the same technique with the spatial positions as the
 * sequence (L = H.W): its backward pass is the linear layer's on the column matrix of the input.
 * All tensors are channels-last, dense, device memory:
 *   X [Nb, H, W, C],  G [Nb, Ho, Wo, O] (= [N, O] with N = Nb*Ho*Wo),  Wt [O, kh, kw, C] (= [O, I]
 *   with I = kh*kw*C),  Ho = (H + 2 pad_h - dil_h (kh-1) - 1) / stride_h + 1, Wo likewise.
 * The geometry is a host struct read during the call.
 */
typedef struct hlq_conv_geom {
    int32_t Nb, H, W, C;                 /* input image batch */
    int32_t O, kh, kw;                   /* filters */
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} hlq_conv_geom;

/* Output extent and the sizes of the equivalent linear layer; HLQ_ERR_SHAPE for a geometry with a
 * non-positive field (sizes, strides, dilations < 1; pads < 0), an empty output, or N, I, W*C, Nb*H or a
 * padded image axis (H + 2 pad_h + kh dil_h, same for W) of 2^31 or more.
 * Any of the output pointers may be NULL. */
int hlq_conv_sizes(const hlq_conv_geom *g, int64_t *Ho, int64_t *Wo, int64_t *N, int64_t *I);

/*
 * Column matrix: cols [N, I], row (n, ho, wo), column (ky, kx, c) -- the order of Wt's trailing
 * axes -- holding X[n, ho stride_h - pad_h + ky dil_h, wo stride_w - pad_w + kx dil_w, c], or 0
 * outside the image.  A pure copy in `dtype`.  X, cols 16-byte aligned.
 */
int hlq_im2col(const void *X, const hlq_conv_geom *g, int dtype, void *cols, void *stream);

/*
 * The adjoint: dX [Nb, H, W, C], each pixel the sum of the entries of cols [N, I] copied from it
 * by hlq_im2col, added in fp32 in ascending (ky, kx) order and rounded once to `dtype`.  Every pixel
 * is written (pixels no output position reads get 0).
 */
int hlq_col2im(const void *cols, const hlq_conv_geom *g, int dtype, void *dX, void *stream);

/*
 * ACBP for a convolution (Sec. 6.1, stage 1 -- and 2 -- of the g_w list at forward time): what
 * hlq_hla_project_basis / hlq_hla_quantize_basis (tensor 2) give on hlq_im2col's result, computed
 * straight from the image -- the column matrix is never stored.  XhatT [I, N/B*r] bf16, or XqT
 * [I, N/B*r] int8 with sX [I]; coeffT as there.  Needs C % (128 / B) == 0 (HLQ_ERR_SHAPE otherwise:
 * store the column matrix and compress that); the other rules and codes are those of the two
 * functions named, with D = I.  The result feeds hlq_linear_backward_mode as Xc (and sXc).
 */
int hlq_conv_compress_act(const void *X, const hlq_conv_geom *g, int B, int r, int basis, int dtype, void *XhatT,
                          float *coeffT, void *stream);
int hlq_conv_compress_act_int8(const void *X, const hlq_conv_geom *g, int B, int r, int basis, uint64_t seed, int dtype,
                               int8_t *XqT, float *sX, float *coeffT, void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * Backward pass of the convolution: hlq_im2col(X), then hlq_linear_backward_mode on (G, cols, Wt)
 * with the N, d_in = I, d_out = O above (same B, r, seed, flags, shape rules and status codes), then
 * hlq_col2im of the column gradient.  dX [Nb, H, W, C] and dW [O, kh, kw, C] of `dtype`; either may
 * be NULL.  A 1x1 kernel with unit stride and no padding is its own column matrix: no copy is made;
 * with C % (128 / B) == 0 the g_w list projects straight from the image (hlq_conv_compress_act) and
 * no column matrix is stored either -- same result bit for bit.  The column gradient is held in
 * `dtype` before it is folded.
 *   workspace >= hlq_conv_workspace_bytes(...) bytes, 256-aligned; or NULL for the library-owned one.
 */
size_t hlq_conv_workspace_bytes(const hlq_conv_geom *g, int B, int r, int dtype, int flags);
int hlq_conv2d_backward(const void *G, const void *X, const void *Wt, const hlq_conv_geom *g, int B, int r,
                        uint64_t seed, int dtype, int flags, void *dX, void *dW, void *workspace,
                        size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HLQ_H_ */
