/*
 * CPU oracle for the batch-reduce matrix multiplication
 *
 *     C = beta * C + sum_{i < batch} A_i (M x K) * B_i (K x N)
 *
 * This file is TEST INFRASTRUCTURE.  It is the slow, plain definition that the
 * GPU library is checked against; nothing in the product path may call it.
 * It shares no code, header, table or helper with the GPU library.
 *
 * What it follows in the paper:
 *   - the input/output statement of Algorithm 1 ("BRGEMM - nanokernels()"):
 *     the result is beta*C plus the sum over the batch of A_i x B_i;
 *   - Section 2.1: the A_i / B_i source tiles need not be contiguous, so every
 *     tile is addressed as base + offset[i];
 *   - Section 5(d): plain matmul is the batch == 1 case;
 *   - the appendix listings with bf16 inputs: each product is formed after
 *     widening both bf16 factors, and summed in a wider type than the inputs;
 *   - Section 4.3 (VNNI-packed paragraph): a bf16 C is widened before
 *     accumulation and narrowed once, after the whole sum, before the store;
 *   - the evaluation's "MLP kernel" (Section 6): bias add and ReLU applied to
 *     the finished sum before the store.
 *
 * Readings taken where the paper is silent:
 *   - beta is an fp32 scalar; beta == 0 means C is never read (so NaN/Inf in
 *     the old C do not propagate);
 *   - there is no alpha (alpha == 1);
 *   - narrowing to bf16 is round-to-nearest-even, NaN -> quiet NaN;
 *   - transA / transB select whether an operand is stored as its logical shape
 *     or transposed, always row-major with an explicit leading dimension.
 *
 * Arithmetic: every input is widened exactly to fp64, every product and sum is
 * fp64 (a bf16*bf16 or fp32*fp32 product is exact in fp64), and beta*C0 is
 * added in fp64.  Loops are the definition written out: no blocking, no
 * reordering beyond choosing which of the three loops is innermost.
 *
 * Pins (tests/test_oracle_pins.py): hand-expanded exact sums with Python
 * integers/fractions, small-integer matrices against int64 arithmetic,
 * identity/permutation matrices, closed forms, associativity, transpose
 * identity, BRGEMM == GEMM on K-concatenated operands, beta linearity, the
 * paper's listing shapes, the bf16 and binary16 helpers against hand-picked bit
 * patterns and a library conversion, and the VNNI packer against Figure 1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

/* bf16 is the upper half of an IEEE-754 binary32; widening is exact. */
static double widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* IEEE-754 binary16 (1 sign, 5 exponent bits with bias 15, 10 fraction bits), the
 * other 16-bit type Section 2.2 names; widening is exact.  Done on values. */
static double widen_f16(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 31)
        v = f ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)f, -24);                  /* subnormal: f * 2^-24 */
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

static double load_elem(const void *p, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16)
        return widen_bf16(((const uint16_t *)p)[idx]);
    if (dtype == ORACLE_F16)
        return widen_f16(((const uint16_t *)p)[idx]);
    return (double)((const float *)p)[idx];
}

/*
 * Round an fp64 value to bf16 (1 sign, 8 exponent, 7 fraction bits) with
 * round-to-nearest, ties-to-even, in one step from the fp64 value.
 * Done on the value, not on bit patterns: scale so that one bf16 quantum is
 * 1.0, round to the nearest integer (ties to even) with rint(), scale back.
 */
uint16_t oracle_f64_to_bf16(double d)
{
    uint16_t sign = signbit(d) ? 0x8000u : 0u;
    if (isnan(d))
        return (uint16_t)(sign | 0x7FC0u);
    double a = fabs(d);
    if (a == 0.0)
        return sign;
    /* Largest finite bf16 is (2 - 2^-7) * 2^127; halfway to the next binade,
     * (2 - 2^-8) * 2^127, already rounds to infinity (its lower neighbour has
     * an odd fraction, so the tie goes up). */
    const double to_inf = ldexp(2.0 - ldexp(1.0, -8), 127);
    if (isinf(d) || a >= to_inf)
        return (uint16_t)(sign | 0x7F80u);
    int e2;
    (void)frexp(a, &e2);        /* a = m * 2^e2, m in [0.5, 1) */
    int E = e2 - 1;             /* a in [2^E, 2^(E+1)) */
    if (E < -126)
        E = -126;               /* subnormal range: fixed quantum */
    int qexp = E - 7;           /* one unit in the last place of bf16 */
    double scaled = ldexp(a, -qexp);   /* exact: power-of-two scaling */
    double r = rint(scaled);           /* default mode: nearest, ties-even */
    float v = (float)ldexp(r, qexp);   /* exactly representable in fp32 */
    uint32_t u;
    memcpy(&u, &v, sizeof u);
    return (uint16_t)(sign | (uint16_t)(u >> 16));
}

double oracle_bf16_to_f64(uint16_t h) { return widen_bf16(h); }

/*
 * Round an fp64 value to binary16 with round-to-nearest, ties-to-even, in one
 * step, the same way as above: one quantum of the target is scaled to 1.0, rint()
 * rounds, and the rounded value is encoded.  Subnormals (quantum 2^-24) are kept;
 * values that round beyond 65504 become infinity; NaN becomes a quiet NaN.
 */
uint16_t oracle_f64_to_f16(double d)
{
    uint16_t sign = signbit(d) ? 0x8000u : 0u;
    if (isnan(d))
        return (uint16_t)(sign | 0x7E00u);
    double a = fabs(d);
    if (a == 0.0)
        return sign;
    /* halfway between 65504 = (2 - 2^-10) * 2^15 and 2^16: ties go to the even
     * neighbour, which is 2^16, i.e. infinity */
    const double to_inf = ldexp(2.0 - ldexp(1.0, -11), 15);
    if (isinf(d) || a >= to_inf)
        return (uint16_t)(sign | 0x7C00u);
    int e2;
    (void)frexp(a, &e2);
    int E = e2 - 1;                     /* a in [2^E, 2^(E+1)) */
    if (E < -14)
        E = -14;                        /* subnormal range: fixed quantum 2^-24 */
    const int qexp = E - 10;
    const double r = rint(ldexp(a, -qexp));      /* integer number of quanta */
    const double v = ldexp(r, qexp);
    if (v == 0.0)
        return sign;
    (void)frexp(v, &e2);
    const int Ev = e2 - 1;              /* may be E + 1 after a carry */
    if (Ev < -14)                       /* subnormal result */
        return (uint16_t)(sign | (uint16_t)ldexp(v, 24));
    const double frac = ldexp(v, -Ev) - 1.0;     /* in [0, 1) */
    return (uint16_t)(sign | (uint16_t)((Ev + 15) << 10) | (uint16_t)ldexp(frac, 10));
}

double oracle_f16_to_f64(uint16_t h) { return widen_f16(h); }

/* Element-wise rounding of an fp64 array to the output type of the GPU
 * library: out_dtype 0 -> fp32 (C cast, round-to-nearest-even), 1 -> bf16,
 * 2 -> binary16. */
void oracle_round_to_out(const double *ref, int64_t count, int out_dtype,
                         void *out)
{
    for (int64_t t = 0; t < count; ++t) {
        if (out_dtype == ORACLE_BF16)
            ((uint16_t *)out)[t] = oracle_f64_to_bf16(ref[t]);
        else if (out_dtype == ORACLE_F16)
            ((uint16_t *)out)[t] = oracle_f64_to_f16(ref[t]);
        else
            ((float *)out)[t] = (float)ref[t];
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * The oracle proper.
 *
 *   in_dtype    element type of every A_i and B_i (ORACLE_F32 / ORACLE_BF16 / ORACLE_F16)
 *   transA      0: A_i stored M x K, element (m,k) at m*lda + k
 *               1: A_i stored K x M, element (m,k) at k*lda + m
 *   transB      0: B_i stored K x N, element (k,n) at k*ldb + n
 *               1: B_i stored N x K, element (k,n) at n*ldb + k
 *   A_off/B_off host arrays of `batch` element offsets from A_base/B_base
 *               (NULL means offset 0 for every i)
 *   beta, C0    old C (c0_dtype, leading dimension ldc0); never read if
 *               beta == 0 (C0 may then be NULL)
 *   bias        NULL, or N fp32 values added to every row of the finished sum
 *   relu        nonzero: negative results become +0 (after beta and bias)
 *   rows/nrows  NULL/0: compute all M rows, ref is M x N dense;
 *               else compute only the listed rows, ref is nrows x N dense
 *
 * Returns 0, or -1 on an argument that makes no sense.
 */
int oracle_brgemm(int in_dtype, int transA, int transB,
                  int64_t M, int64_t N, int64_t K, int64_t batch,
                  const void *A_base, const int64_t *A_off, int64_t lda,
                  const void *B_base, const int64_t *B_off, int64_t ldb,
                  float beta, const void *C0, int c0_dtype, int64_t ldc0,
                  const float *bias, int relu,
                  const int64_t *rows, int64_t nrows,
                  double *ref)
{
    if (M < 0 || N < 0 || K < 0 || batch < 0 || !ref)
        return -1;
    if (beta != 0.0f && !C0 && M > 0 && N > 0)
        return -1;
    int64_t R = rows ? nrows : M;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < R; ++r) {
        int64_t m = rows ? rows[r] : r;
        double *acc = ref + r * N;
        if (m < 0 || m >= M) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        for (int64_t n = 0; n < N; ++n)
            acc[n] = 0.0;

        for (int64_t i = 0; i < batch; ++i) {
            int64_t ao = A_off ? A_off[i] : 0;
            int64_t bo = B_off ? B_off[i] : 0;
            if (!transB) {
                /* B_i row k is contiguous: run k outside, n inside. */
                for (int64_t k = 0; k < K; ++k) {
                    double a = load_elem(A_base, in_dtype,
                                         ao + (transA ? k * lda + m : m * lda + k));
                    for (int64_t n = 0; n < N; ++n)
                        acc[n] += a * load_elem(B_base, in_dtype, bo + k * ldb + n);
                }
            } else {
                /* B_i stored N x K: column n of B_i is contiguous in k. */
                for (int64_t n = 0; n < N; ++n) {
                    double s = 0.0;
                    for (int64_t k = 0; k < K; ++k) {
                        double a = load_elem(A_base, in_dtype,
                                             ao + (transA ? k * lda + m : m * lda + k));
                        s += a * load_elem(B_base, in_dtype, bo + n * ldb + k);
                    }
                    acc[n] += s;
                }
            }
        }

        for (int64_t n = 0; n < N; ++n) {
            double v = acc[n];
            if (beta != 0.0f)
                v += (double)beta * load_elem(C0, c0_dtype, m * ldc0 + n);
            if (bias)
                v += (double)bias[n];
            if (relu && v < 0.0)
                v = 0.0;
            acc[n] = v;
        }
    }
    return bad ? -1 : 0;
}

/*
 * VNNI packing of the B operand (Section 2.2 and Figure 1): the K dimension is cut
 * into groups of v consecutive rows and the v elements of one column within a
 * group are stored next to each other,
 *
 *     out[(k / v) * n_pitch * v + n * v + (k % v)] = B[k][n],
 *
 * which turns a K x N matrix into a (K / v) x N x v one (Figure 1: a flat 4 x 4
 * matrix becomes 2 x 4 x 2 for v = 2).  B is read through transB / ldb like the
 * GEMM operand (transB == 1: stored N x K).  The output has k_rows rows of k
 * (k_rows >= K, a multiple of v) and n_pitch >= N columns per group; everything
 * that does not come from B (rows K.., columns N..) is zero.  Elements are 16-bit
 * patterns and are moved, never converted.
 * Returns 0, or -1 on a bad argument.
 */
int oracle_pack_vnni(int v, int transB, int64_t K, int64_t N, const uint16_t *B, int64_t ldb,
                     int64_t k_rows, int64_t n_pitch, uint16_t *out)
{
    if (v <= 0 || K < 0 || N < 0 || k_rows < K || k_rows % v != 0 || n_pitch < N)
        return -1;
    for (int64_t i = 0; i < k_rows * n_pitch; ++i)
        out[i] = 0;
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n) {
            const uint16_t e = transB ? B[n * ldb + k] : B[k * ldb + n];
            out[(k / v) * n_pitch * v + n * v + (k % v)] = e;
        }
    return 0;
}

/*
 * int8 matrix multiplication with exact integer accumulation (Section 2.2 names INT8
 * among the packed types; Section 5(c): other types follow the same structure):
 *
 *     out[m][n] = (accumulate ? C0[m][n] : 0) + sum_k A(m,k) * B(k,n)
 *
 * A and B are signed 8-bit, read through transA / transB / lda / ldb exactly as in
 * oracle_brgemm; C0 is int32; the sum is formed in int64 (no wrap-around is possible
 * for K < 2^31) and returned as int64, so a 32-bit overflow of the true result shows
 * up as a value outside the int32 range rather than being hidden.
 * Returns 0, or -1 on a bad argument.
 */
int oracle_gemm_s8(int transA, int transB, int64_t M, int64_t N, int64_t K,
                   const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                   int accumulate, const int32_t *C0, int64_t ldc0, int64_t *out)
{
    if (M < 0 || N < 0 || K < 0 || (accumulate && !C0))
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = accumulate ? (int64_t)C0[m * ldc0 + n] : 0;
            for (int64_t k = 0; k < K; ++k) {
                const int64_t a = transA ? A[k * lda + m] : A[m * lda + k];
                const int64_t b = transB ? B[n * ldb + k] : B[k * ldb + n];
                s += a * b;
            }
            out[m * N + n] = s;
        }
    return 0;
}

/*
 * FP8 operands (Section 5(c): further packed types follow the same structure; the 8-bit
 * float of the OCP "E4M3" kind: 1 sign, 4 exponent bits with bias 7, 3 fraction bits, no
 * infinities, the single NaN pattern S.1111.111, largest finite value 448).  Decoded on
 * values, exactly; the product of the widened operands is then the oracle above with fp32
 * inputs, since every E4M3 value is exactly representable in fp32.
 */
double oracle_f8e4m3_to_f64(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 3) & 15, f = b & 7;
    double v;
    if (e == 15 && f == 7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)f, -9);                    /* subnormal: f/8 * 2^-6 */
    else
        v = ldexp(1.0 + (double)f / 8.0, e - 7);
    return sign ? -v : v;
}

/* Widen `count` E4M3 bytes to fp32 (exact). */
void oracle_f8e4m3_widen(const uint8_t *src, int64_t count, float *dst)
{
    for (int64_t i = 0; i < count; ++i)
        dst[i] = (float)oracle_f8e4m3_to_f64(src[i]);
}

/*
 * The other 8-bit float of the same family (OCP "E5M2": 1 sign, 5 exponent bits with bias
 * 15, 2 fraction bits; exponent 31 holds the infinities (fraction 0) and NaN (fraction
 * != 0), largest finite value 57344, subnormals f/4 * 2^-14).  Section 5(c) again: one
 * more packed type through the same structure.  Decoded on values, exactly; every E5M2
 * value is exactly representable in fp32 (and in binary16, whose top byte it is).
 */
double oracle_f8e5m2_to_f64(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 2) & 31, f = b & 3;
    double v;
    if (e == 31)
        v = f ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)f, -16);                   /* subnormal: f/4 * 2^-14 */
    else
        v = ldexp(1.0 + (double)f / 4.0, e - 15);
    return sign ? -v : v;
}

/* Widen `count` E5M2 bytes to fp32 (exact). */
void oracle_f8e5m2_widen(const uint8_t *src, int64_t count, float *dst)
{
    for (int64_t i = 0; i < count; ++i)
        dst[i] = (float)oracle_f8e5m2_to_f64(src[i]);
}
