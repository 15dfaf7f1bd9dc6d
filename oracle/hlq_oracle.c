/*
 * HLQ backward-pass oracle  --  TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, CPU-only statement of what the Hadamard Low-rank Quantization
 * (HLQ) backward pass of a linear layer computes, written from the paper
 * (arXiv 2406.15102) step by step in the paper's order.  Only the test-suite,
 * the smoke check and the benchmark's CPU-baseline leg may call it.  It shares
 * no code, table or helper with the HIP library and must never be reached from
 * the product path.
 *
 * Conventions (paper notation -> here):
 *   tokens  (paper B*L, Sec. 3.1)  -> N        in-features  (paper I) -> d_in
 *   Hadamard order (paper n, Sec. 6.1, = 16)   -> B           out-features (paper O) -> d_out
 *   kept bases (paper r, = 8)      -> r
 *   G  = g_y reshaped to [N, d_out],  X = x reshaped to [N, d_in],  W = w [d_out, d_in]
 *   (Sec. 3.1, Eq. 1).  All matrices are dense row-major.
 *
 * What is computed:
 *   g_x path (Sec. 5.1 and the six g_x stages of Sec. 6.1):
 *     dX = Q(G H_O) . Q(H_O^T W)        block-diagonal H along the out-feature axis
 *   g_w path (Sec. 5.1 and stages 1,3,5 of the six g_w stages of Sec. 6.1, kept in bf16):
 *     dW = (G^T H_L^T)(H_L X)           block-diagonal H along the token axis, r of B bases kept
 *
 * Readings of points the paper leaves open (each one is restated where used):
 *   - H is the +-1 Sylvester matrix (Eq. 2 without the 1/sqrt(2) per level); the
 *     normalisation is applied once as an exact 1/B at the end of each path.
 *   - "min-max" 4-bit quantiser (Sec. 5.1, 6.1): symmetric absmax, codes in
 *     [-7, 7], one scale per row of the reduction-contiguous operand.
 *   - stochastic rounding (Sec. 6.1) draws its bits from a seeded counter-based
 *     generator instead of the low mantissa bits of the data.
 *   - the r kept bases are rows 0..r-1 of the natural-order Sylvester matrix.
 *   - Eq. 1's 1/B_batch factor is left to the caller (G carries it).
 *
 * Precision: coefficients that decide integer codes are fp32 sums in a fixed
 * balanced pairwise order (so that an integer decision has one right answer);
 * everything that does not decide an integer is fp64.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py
 * against closed forms, library routines or brute force; nothing here is
 * pinned to numbers printed in the paper (it prints none for these kernels):
 * "parity against the paper's own numbers: unpinned".
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC hlq_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define HLQO_MAX_B 64

int hlqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Walsh-Hadamard matrix (Sec. 3.2, Eq. 2): H_2 = [[1,1],[1,-1]],             */
/* H_{2m} = H_2 (x) H_m, built by the Kronecker recursion itself, entries +-1. */
/* Returns 0, or -1 when B is not a power of two in [1, 64].                  */
/* ------------------------------------------------------------------------- */
int hlqo_hadamard(int B, int8_t *H /* [B*B] */)
{
    if (B < 1 || B > HLQO_MAX_B || (B & (B - 1)) != 0) return -1;
    H[0] = 1;
    for (int m = 1; m < B; m *= 2) {
        /* grow the m x m matrix held in the top-left corner (row pitch B) to 2m x 2m */
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < m; ++j) {
                int8_t h = H[i * B + j];
                H[i * B + (j + m)] = h;        /* [ H  H ] */
                H[(i + m) * B + j] = h;        /* [ H -H ] */
                H[(i + m) * B + (j + m)] = (int8_t)-h;
            }
    }
    return 0;
}

/* Balanced pairwise sum of t[lo..hi) in natural index order; every + is one   */
/* IEEE binary32 round-to-nearest-even addition.                               */
static float pairwise_sum_f32(const float *t, int lo, int hi)
{
    if (hi - lo == 1) return t[lo];
    int mid = (lo + hi) / 2;
    float a = pairwise_sum_f32(t, lo, mid);
    float b = pairwise_sum_f32(t, mid, hi);
    return a + b;
}

/* One Hadamard coefficient block: c_i = sum_j H[i][j] v[j*stride], i < nout.  */
/* The products are exact sign flips; the sum is the pairwise sum above.       */
/* This is the explicit matrix-vector product of Sec. 3.2, not an FWHT.        */
static void coeff_f32(const int8_t *H, int B, const float *v, long stride, int nout, float *c)
{
    float t[HLQO_MAX_B];
    for (int i = 0; i < nout; ++i) {
        for (int j = 0; j < B; ++j) t[j] = (H[i * B + j] > 0) ? v[j * stride] : -v[j * stride];
        c[i] = pairwise_sum_f32(t, 0, B);
    }
}

/* Same coefficients in fp64, summed left to right (the value the fp32 ones approximate). */
static void coeff_f64(const int8_t *H, int B, const float *v, long stride, int nout, double *c)
{
    for (int i = 0; i < nout; ++i) {
        double s = 0.0;
        for (int j = 0; j < B; ++j) s += (double)H[i * B + j] * (double)v[j * stride];
        c[i] = s;
    }
}

int hlqo_coeff_f32(int B, const float *v, long stride, int nout, float *c)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || nout < 0 || nout > B) return -1;
    coeff_f32(H, B, v, stride, nout, c);
    return 0;
}

int hlqo_coeff_f64(int B, const float *v, long stride, int nout, double *c)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || nout < 0 || nout > B) return -1;
    coeff_f64(H, B, v, stride, nout, c);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Block-diagonal transform (Sec. 3.2, last paragraph) along the out-feature  */
/* axis: stage 1 and stage 3 of the g_x path (Sec. 6.1).                      */
/* ------------------------------------------------------------------------- */

/* Ghat[n, b*B + i] = c_i( G[n, b*B .. b*B+B) )           (g_y . H_O)          */
int hlqo_transform_rows(const float *G, long N, long O, int B, float *Ghat /* [N,O] */)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || O % B) return -1;
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n)
        for (long b = 0; b < O / B; ++b)
            coeff_f32(H, B, G + n * O + b * B, 1, B, Ghat + n * O + b * B);
    return 0;
}

/* WhatT[col, b*B + i] = c_i( W[b*B .. b*B+B, col] )      (H_O^T . w), stored   */
/* transposed so that the reduction axis (out-features) is contiguous.         */
int hlqo_transform_cols(const float *W, long O, long I, int B, float *WhatT /* [I,O] */)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || O % B) return -1;
#pragma omp parallel for schedule(static)
    for (long col = 0; col < I; ++col)
        for (long b = 0; b < O / B; ++b)
            coeff_f32(H, B, W + b * B * I + col, I, B, WhatT + col * O + b * B);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Seeded counter-based random bits for stochastic rounding (Sec. 6.1 asks    */
/* for an unbiased stochastic quantiser; the generator is this build's).      */
/* ------------------------------------------------------------------------- */

/* Stream key for (seed, tensor id): output number (tensor+1) of the SplitMix64 */
/* generator (Steele, Lea, Flood 2014; Vigna's public-domain constants)         */
/* started at state = seed.  tensor: 0 = G operand, 1 = W operand of the g_x     */
/* product; 2 = projected X, 3 = projected G of the integer g_w product.         */
uint64_t hlqo_stream_key(uint64_t seed, uint32_t tensor)
{
    uint64_t z = seed + ((uint64_t)tensor + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* 32-bit word number `counter` of the stream `key`: a keyed xorshift-multiply */
/* bijection of the counter (multipliers of Wellons' "lowbias32" integer hash, */
/* public domain), the low key half xored in before, the high half between the */
/* two multiplies.                                                             */
uint32_t hlqo_rand_word(uint64_t key, uint32_t counter)
{
    uint32_t x = counter ^ (uint32_t)key;
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x ^= (uint32_t)(key >> 32);
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

/* Random byte for element (row, pos) of an operand with `K` positions per row: */
/* word counter = row*(K/4) + pos/4, byte (pos mod 4) of that word.             */
uint32_t hlqo_rand_byte(uint64_t key, long row, long pos, long K)
{
    uint32_t counter = (uint32_t)((uint64_t)row * (uint64_t)(K / 4) + (uint64_t)(pos / 4));
    return (hlqo_rand_word(key, counter) >> (8 * (pos & 3))) & 0xFFu;
}

/* ------------------------------------------------------------------------- */
/* Stochastic "min-max" quantiser (Sec. 5.1, Sec. 6.1): stages 2 and 4 of the  */
/* g_x path with 4-bit codes (qmax = 7), and with qmax = 127 the int8          */
/* quantiser of stages 2 and 4 of the g_w path and of the 8-bit warm-up phase  */
/* (Sec. 7, "all quantization operators use int8 at the initial 25 epochs").   */
/*   a     = max_k |C[row,k]|             per row                              */
/*   inv   = qmax/a (0 when a == 0),  scale = a/qmax                           */
/*   u     = (byte + 0.5)/256   in (0,1), uniform                              */
/*   q     = clamp(floor(x*inv + u), -qmax, qmax)   x*inv+u rounded once (fma) */
/* floor(y + u) with u uniform on (0,1) rounds y up with probability frac(y):  */
/* the unbiased stochastic rounding the paper requires.                        */
/* ------------------------------------------------------------------------- */
int8_t hlqo_quantize_one_q(float x, float inv, uint32_t byte, int qmax)
{
    float u = ((float)byte + 0.5f) * 0.00390625f;
    float t = fmaf(x, inv, u);
    int q = (int)floorf(t);
    if (q > qmax) q = qmax;
    if (q < -qmax) q = -qmax;
    return (int8_t)q;
}

int8_t hlqo_quantize_one(float x, float inv, uint32_t byte) { return hlqo_quantize_one_q(x, inv, byte, 7); }

/* Quantise `rows` rows of C; row_ids[i] (or i when row_ids is NULL) is the row's index in the   */
/* full operand, which is what addresses its random bytes: a subset of rows gets the same codes */
/* it has inside the full matrix.  qmax is 7 (4-bit codes) or 127 (8-bit codes).                */
int hlqo_quantize_rows_q(const float *C, long rows, long K, uint64_t seed, uint32_t tensor,
                         const long *row_ids, int qmax, int8_t *q /* [rows,K] */, float *scale /* [rows] */)
{
    if (K % 4 || (qmax != 7 && qmax != 127)) return -1;
    uint64_t key = hlqo_stream_key(seed, tensor);
    const float fq = (float)qmax;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const long row = row_ids ? row_ids[i] : i;
        const float *c = C + i * K;
        float a = 0.0f;
        for (long k = 0; k < K; ++k) {
            float m = fabsf(c[k]);
            if (m > a) a = m;
        }
        float inv = (a > 0.0f) ? fq / a : 0.0f;
        scale[i] = a / fq;
        for (long k = 0; k < K; ++k)
            q[i * K + k] = hlqo_quantize_one_q(c[k], inv, hlqo_rand_byte(key, row, k, K), qmax);
    }
    return 0;
}

/* The paper's own source of rounding randomness (Sec. 6.1): "the lower 11 bits of floating-point   */
/* data" of the value being quantised stand in for the random number, at no generation cost:      */
/*   m = low 11 bits of the binary32 pattern of x,   u = (m + 0.5)/2048,   q = floor(x*inv + u)   */
/* Nothing else changes.  It is only as random as those bits are: for values that carry fewer    */
/* than 24 significant bits (sums of a few bf16 numbers) they are mostly zero and the quantiser   */
/* degenerates to rounding down.                                                                  */
int8_t hlqo_quantize_one_mantissa(float x, float inv, int qmax)
{
    uint32_t bits;
    memcpy(&bits, &x, 4);
    float u = ((float)(bits & 0x7FFu) + 0.5f) * 0.00048828125f;   /* / 2048, exact */
    float t = fmaf(x, inv, u);
    int q = (int)floorf(t);
    if (q > qmax) q = qmax;
    if (q < -qmax) q = -qmax;
    return (int8_t)q;
}

int hlqo_quantize_rows_mantissa(const float *C, long rows, long K, int qmax, int8_t *q /* [rows,K] */,
                                float *scale /* [rows] */)
{
    if (qmax != 7 && qmax != 127) return -1;
    const float fq = (float)qmax;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const float *c = C + i * K;
        float a = 0.0f;
        for (long k = 0; k < K; ++k) {
            float m = fabsf(c[k]);
            if (m > a) a = m;
        }
        float inv = (a > 0.0f) ? fq / a : 0.0f;
        scale[i] = a / fq;
        for (long k = 0; k < K; ++k) q[i * K + k] = hlqo_quantize_one_mantissa(c[k], inv, qmax);
    }
    return 0;
}

int hlqo_quantize_rows_at(const float *C, long rows, long K, uint64_t seed, uint32_t tensor,
                          const long *row_ids, int8_t *q, float *scale)
{
    return hlqo_quantize_rows_q(C, rows, K, seed, tensor, row_ids, 7, q, scale);
}

int hlqo_quantize_rows(const float *C, long rows, long K, uint64_t seed, uint32_t tensor,
                       int8_t *q /* [rows,K] */, float *scale /* [rows] */)
{
    return hlqo_quantize_rows_q(C, rows, K, seed, tensor, NULL, 7, q, scale);
}

/* ------------------------------------------------------------------------- */
/* Stage 5 of the g_x path: integer matrix product, exact in int32.            */
/* acc[m, n] = sum_k A[m,k] * Bm[n,k]                                          */
/* ------------------------------------------------------------------------- */
int hlqo_int_gemm_nt(const int8_t *A, const int8_t *Bm, long M, long Nn, long K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (long n = 0; n < Nn; ++n) {
            int32_t s = 0;
            for (long k = 0; k < K; ++k) s += (int32_t)A[m * K + k] * (int32_t)Bm[n * K + k];
            acc[m * Nn + n] = s;
        }
    return 0;
}

/* Stage 6 of the g_x path: dequantise.  The two scales undo the quantiser and */
/* 1/B undoes the unnormalised H.H^T = B.I.  fp64, no rounding to the output   */
/* type here.                                                                  */
int hlqo_dequant(const int32_t *acc, const float *sA, const float *sB, long M, long Nn, int B,
                 double *out)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (long n = 0; n < Nn; ++n)
            out[m * Nn + n] = (double)acc[m * Nn + n] * (double)sA[m] * (double)sB[n] / (double)B;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Hadamard low-rank approximation along the token axis (Sec. 4, Sec. 5.1;     */
/* stages 1 and 3 of the g_w path, Sec. 6.1; stage 1 is also what ACBP stores  */
/* at forward time).  For token block b and column j:                          */
/*   ChatT[j, b*r + k] = c_k( T[b*B .. b*B+B, j] ),  k < r                      */
/* stored with the compressed token axis contiguous.  fp32 (same pairwise sum) */
/* and fp64 versions.                                                          */
/* ------------------------------------------------------------------------- */
/* Which rows of H are "the first r".  basis 0: rows 0..r-1 as Eq. 2 numbers them (natural order).     */
/* basis 1: the r rows of lowest SEQUENCY, in order of increasing sequency, where the sequency of a     */
/* row is the number of sign changes along it -- the Walsh functions' analogue of frequency, which is  */
/* what "low-frequency components" of g_w (Sec. 4) and the low-pass base selection of LBP-WHT (Sec.     */
/* 6.1) refer to.  The rows are found from that definition: count the sign changes of every row.       */
int hlqo_basis_rows(int B, int basis, int *rows /* [B] */)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || (basis != 0 && basis != 1)) return -1;
    for (int k = 0; k < B; ++k) rows[k] = -1;
    for (int n = 0; n < B; ++n) {
        int changes = 0;
        for (int j = 1; j < B; ++j) changes += H[n * B + j] != H[n * B + j - 1];
        int k = basis ? changes : n;
        if (rows[k] != -1) return -1;   /* the sequencies of the B rows are 0..B-1, each once */
        rows[k] = n;
    }
    return 0;
}

/* coefficient of one given row of H: the one-row case of coeff_f32 / coeff_f64 */
static float coeff_row_f32(const int8_t *H, int B, int row, const float *v, long stride)
{
    float c;
    coeff_f32(H + row * B, B, v, stride, 1, &c);
    return c;
}

static double coeff_row_f64(const int8_t *H, int B, int row, const float *v, long stride)
{
    double c;
    coeff_f64(H + row * B, B, v, stride, 1, &c);
    return c;
}

int hlqo_hla_basis_f32(const float *T, long N, long D, int B, int r, int basis, float *ChatT /* [D, N/B*r] */)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    int rows[HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || hlqo_basis_rows(B, basis, rows) || N % B || r < 1 || r > B) return -1;
    long Kc = N / B * r;
#pragma omp parallel for schedule(static)
    for (long j = 0; j < D; ++j)
        for (long b = 0; b < N / B; ++b)
            for (int k = 0; k < r; ++k)
                ChatT[j * Kc + b * r + k] = coeff_row_f32(H, B, rows[k], T + b * B * D + j, D);
    return 0;
}

int hlqo_hla_basis_f64(const float *T, long N, long D, int B, int r, int basis, double *ChatT /* [D, N/B*r] */)
{
    int8_t H[HLQO_MAX_B * HLQO_MAX_B];
    int rows[HLQO_MAX_B];
    if (hlqo_hadamard(B, H) || hlqo_basis_rows(B, basis, rows) || N % B || r < 1 || r > B) return -1;
    long Kc = N / B * r;
#pragma omp parallel for schedule(static)
    for (long j = 0; j < D; ++j)
        for (long b = 0; b < N / B; ++b)
            for (int k = 0; k < r; ++k)
                ChatT[j * Kc + b * r + k] = coeff_row_f64(H, B, rows[k], T + b * B * D + j, D);
    return 0;
}

int hlqo_hla_f32(const float *T, long N, long D, int B, int r, float *ChatT /* [D, N/B*r] */)
{
    return hlqo_hla_basis_f32(T, N, D, B, r, 0, ChatT);
}

int hlqo_hla_f64(const float *T, long N, long D, int B, int r, double *ChatT /* [D, N/B*r] */)
{
    return hlqo_hla_basis_f64(T, N, D, B, r, 0, ChatT);
}

/* Round an fp32 value to the nearest bfloat16 (ties to even), returned as the */
/* fp32 value it denotes.  bfloat16 = the top 16 bits of binary32.             */
float hlqo_round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return x; /* inf / nan unchanged */
    uint32_t keep = u & 0xFFFF0000u;
    uint32_t rest = u & 0x0000FFFFu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 0x00010000u))) keep += 0x00010000u;
    float y;
    memcpy(&y, &keep, 4);
    return y;
}

void hlqo_round_bf16_array(const float *x, long n, float *y)
{
    for (long i = 0; i < n; ++i) y[i] = hlqo_round_bf16(x[i]);
}

/* Stage 5 of the g_w path: out[m, n] = alpha * sum_k A[m,k] * Bm[n,k], fp64.   */
int hlqo_gemm_nt_f64(const float *A, const float *Bm, long M, long Nn, long K, double alpha,
                     double *out)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (long n = 0; n < Nn; ++n) {
            double s = 0.0;
            for (long k = 0; k < K; ++k) s += (double)A[m * K + k] * (double)Bm[n * K + k];
            out[m * Nn + n] = alpha * s;
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The whole backward pass, composed from the stages above in the paper's      */
/* order.  Inputs are fp32 arrays (bf16 data is passed widened, which is       */
/* exact).  Outputs are fp64; rounding to the caller's output type is the      */
/* caller's last step.  Optional outputs may be NULL.                          */
/*   dX  [N, d_in]    dW [d_out, d_in]                                          */
/*   Gq  [N, d_out] int8, sG [N], Wq [d_in, d_out] int8, sW [d_in]              */
/*   acc [N, d_in] int32                                                        */
/*   GhatT [d_out, N/B*r], XhatT [d_in, N/B*r]: bf16-rounded HLA coefficients   */
/* Returns 0, -1 on a shape error, -2 when out of memory.                       */
/* ------------------------------------------------------------------------- */
int hlqo_linear_backward(const float *G, const float *X, const float *W, long N, long d_in,
                         long d_out, int B, int r, uint64_t seed, double *dX, double *dW,
                         int8_t *Gq_out, float *sG_out, int8_t *Wq_out, float *sW_out,
                         int32_t *acc_out, float *GhatT_out, float *XhatT_out)
{
    if (N <= 0 || d_in <= 0 || d_out <= 0 || d_out % B || N % B || r < 1 || r > B || d_out % 4)
        return -1;
    int rc = -2;
    long Kc = N / B * r;
    float *coef = NULL, *sG = NULL, *sW = NULL, *gh = NULL, *xh = NULL;
    int8_t *Gq = NULL, *Wq = NULL;
    int32_t *acc = NULL;

    if (dX) {
        /* g_x path, Sec. 6.1: 1. FWH(g_o) on O  2. Q4  3. FWH(w) on O  4. Q4  5. int GEMM  6. dequant */
        long big = (N > d_in ? N : d_in) * d_out;
        coef = (float *)malloc(sizeof(float) * (size_t)big);
        Gq = (int8_t *)malloc((size_t)(N * d_out));
        Wq = (int8_t *)malloc((size_t)(d_in * d_out));
        sG = (float *)malloc(sizeof(float) * (size_t)N);
        sW = (float *)malloc(sizeof(float) * (size_t)d_in);
        acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N * d_in));
        if (!coef || !Gq || !Wq || !sG || !sW || !acc) goto done;
        if (hlqo_transform_rows(G, N, d_out, B, coef)) { rc = -1; goto done; }
        hlqo_quantize_rows(coef, N, d_out, seed, 0u, Gq, sG);
        if (hlqo_transform_cols(W, d_out, d_in, B, coef)) { rc = -1; goto done; }
        hlqo_quantize_rows(coef, d_in, d_out, seed, 1u, Wq, sW);
        hlqo_int_gemm_nt(Gq, Wq, N, d_in, d_out, acc);
        hlqo_dequant(acc, sG, sW, N, d_in, B, dX);
        if (Gq_out) memcpy(Gq_out, Gq, (size_t)(N * d_out));
        if (Wq_out) memcpy(Wq_out, Wq, (size_t)(d_in * d_out));
        if (sG_out) memcpy(sG_out, sG, sizeof(float) * (size_t)N);
        if (sW_out) memcpy(sW_out, sW, sizeof(float) * (size_t)d_in);
        if (acc_out) memcpy(acc_out, acc, sizeof(int32_t) * (size_t)(N * d_in));
    }
    if (dW) {
        /* g_w path, Sec. 6.1 stages 1, 3, 5 (the int8 stages 2, 4, 6 are not applied:  */
        /* the projected operands are rounded to bf16 instead) */
        gh = (float *)malloc(sizeof(float) * (size_t)(d_out * Kc));
        xh = (float *)malloc(sizeof(float) * (size_t)(d_in * Kc));
        if (!gh || !xh) goto done;
        if (hlqo_hla_f32(X, N, d_in, B, r, xh)) { rc = -1; goto done; }
        if (hlqo_hla_f32(G, N, d_out, B, r, gh)) { rc = -1; goto done; }
        hlqo_round_bf16_array(xh, d_in * Kc, xh);
        hlqo_round_bf16_array(gh, d_out * Kc, gh);
        hlqo_gemm_nt_f64(gh, xh, d_out, d_in, Kc, 1.0 / (double)B, dW);
        if (GhatT_out) memcpy(GhatT_out, gh, sizeof(float) * (size_t)(d_out * Kc));
        if (XhatT_out) memcpy(XhatT_out, xh, sizeof(float) * (size_t)(d_in * Kc));
    }
    rc = 0;
done:
    free(coef); free(Gq); free(Wq); free(sG); free(sW); free(acc); free(gh); free(xh);
    return rc;
}
