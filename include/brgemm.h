/*
 * brgemm.h - C ABI of the MI355X (gfx950) GEMM / batch-reduce GEMM library.
 *
 * The operation is the one stated as input/output of Algorithm 1
 * ("BRGEMM - nanokernels()") of the paper:
 *
 *        C  =  beta * C  +  sum_{i=0}^{batch-1}  A_i (M x K)  x  B_i (K x N)
 *
 * with plain matrix multiplication as its batch == 1 case (Section 5(d)).
 * There is no alpha.  beta is an fp32 scalar; beta == 0 means C is written
 * without ever being read, so NaN or Inf in the old C do not propagate.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All matrices are row-major.  ldX is the number of ELEMENTS between the
 *    starts of two consecutive stored rows (>= the stored row length).
 *  - transA == 0: A_i is stored as M x K;  transA == 1: stored as K x M.
 *    transB == 0: B_i is stored as K x N;  transB == 1: stored as N x K
 *    (the usual "NT" weight layout).  Section 4.3 ("Flat Layout") is the
 *    passage that says which operand needs re-laying-out for which storage
 *    order; here both orders of both operands are accepted.
 *  - Every pointer is a DEVICE pointer (hipMalloc / torch CUDA tensor), unless
 *    the argument says "host".  The caller owns every buffer.  The library never
 *    allocates, frees or synchronises: work is enqueued on `stream` (a
 *    hipStream_t passed as void*, NULL = the default stream) and the call
 *    returns at once.  C must not overlap A, B or the workspace.  A_i / B_i
 *    tiles may overlap one another (they are only read).
 *  - Any M, N, K, batch >= 0 and any alignment is accepted.  M == 0 or N == 0
 *    is a no-op.  K == 0 or batch == 0 gives C = beta * C.  The tuned kernels are
 *    taken when bases/offsets are 16-byte aligned and the leading dimensions
 *    are multiples of 8 (bf16) or 4 (fp32) elements; anything else runs on a
 *    slower general kernel with the same results.
 *  - `workspace` may be NULL (workspace_bytes == 0): then no variant that
 *    splits the reduction over several workgroups is chosen.  When given it
 *    must be 256-byte aligned; gemm_workspace_bytes() returns a size that is
 *    always enough.  Its contents before and after a call are unspecified.
 *    Two calls that share a workspace must be ordered on one stream.
 *  - Return value: 0 on success, a negative BRGEMM_* code otherwise.  Nothing
 *    is launched when an argument is rejected.  No exception or abort crosses
 *    this boundary.
 *  - Thread safety: calls may be made concurrently from several host threads.
 *
 * Arithmetic: bf16 factors are widened exactly, products and sums are fp32
 * (the appendix listings of the paper: widen, multiply, add into an f32
 * accumulator); the accumulator tile stays in registers across the whole K and
 * batch loops (Section 2.1, advantage (1)); beta*C and the optional bias are
 * added in fp32; a bf16 C is widened on read and narrowed once, with
 * round-to-nearest-even, on the final store (Section 4.3, VNNI-packed
 * paragraph).  The order of the fp32 summation is unspecified.
 */
#ifndef BRGEMM_H
#define BRGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    BRGEMM_OK = 0,
    BRGEMM_INVALID_ARG = -1,         /* negative size, ld too small, bad flag, NULL operand   */
    BRGEMM_UNSUPPORTED = -2,         /* reserved; no currently accepted input returns it      */
    BRGEMM_WORKSPACE_TOO_SMALL = -3, /* a forced split variant needs more workspace           */
    BRGEMM_HIP_ERROR = -4,           /* launch failed; see gemm_last_hip_error()              */
    BRGEMM_MISALIGNED_WORKSPACE = -5,
    BRGEMM_SCRATCH_TOO_SMALL = -6    /* gemm_bf16_noalloc: split partial sums exceed its buffer */
};

/* Element types, for gemm_workspace_bytes(). */
enum { BRGEMM_DTYPE_F32 = 0, BRGEMM_DTYPE_BF16 = 1, BRGEMM_DTYPE_F16 = 2 };

/* Epilogue flags (Section 6: the measured "MLP kernel" fuses bias and ReLU
 * before the store of the accumulator). */
enum { BRGEMM_EPI_NONE = 0, BRGEMM_EPI_BIAS = 1, BRGEMM_EPI_RELU = 2 };

/*
 * fp32 GEMM:  C[M,N] = beta*C + A[M,K] x B[K,N]   (Algorithm 1, f32 branch).
 * A, B, C: device, fp32.  lda/ldb/ldc in elements.
 */
int gemm_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
             const float *A, int64_t lda, const float *B, int64_t ldb,
             float beta, float *C, int64_t ldc,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * bf16 GEMM with fp32 accumulation (Algorithm 1, bf16 branches; both storage
 * orders of B are the paper's "Flat" layout, no pre-packing is required).
 * A, B: device, bf16 bit patterns.  C: device; fp32 if c_is_f32 != 0, else
 * bf16 (widened on read when beta != 0, rounded to nearest-even on store).
 */
int gemm_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K,
              const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
              float beta, void *C, int64_t ldc, int c_is_f32,
              void *workspace, size_t workspace_bytes, void *stream);

/*
 * gemm_bf16 for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same operation, arguments, plan and results as gemm_bf16 called with a
 * workspace of gemm_workspace_bytes(); the partial sums of a reduction split (skinny-M
 * and small-grid shapes) go to a buffer that is part of the library's code object,
 * BRGEMM_NOALLOC_SCRATCH_BYTES of device memory per GPU, held until the process ends.
 * The call makes no hipMalloc / hipFree and calls no allocating routine.  A problem
 * whose plan needs split * M * N * 4 bytes beyond that size is refused with
 * BRGEMM_SCRATCH_TOO_SMALL and nothing is launched (M = 128, N = 11008 needs 11 MiB;
 * problems that run unsplit, such as 4096^3, need none and are always accepted).
 * The first call on a device looks the buffer's address up (make one call before
 * starting a graph capture).  All calls on one GPU share the buffer: calls that may
 * overlap there (different streams, different host threads) race; order them on one
 * stream.  Its contents are overwritten by every split call and need no clearing.
 */
#define BRGEMM_NOALLOC_SCRATCH_BYTES (32u << 20)
int gemm_bf16_noalloc(int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                      float beta, void *C, int64_t ldc, int c_is_f32, void *stream);

/*
 * The same for IEEE binary16 operands (Section 2.2 names FP16 beside BF16 among
 * the mixed-precision types; Section 5(c): other packed types follow the same
 * structure).  A, B: device, binary16 bit patterns; products and sums are fp32;
 * C is fp32 if c_is_f32 != 0, else binary16 (widened on read, rounded to
 * nearest-even once on store, subnormals kept, overflow to infinity).
 */
int gemm_f16(int transA, int transB, int64_t M, int64_t N, int64_t K,
             const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
             float beta, void *C, int64_t ldc, int c_is_f32,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * FP8 GEMM (Section 5(c): further packed types follow the same structure).  A, B:
 * device, one byte per element in the OCP E4M3 format (1 sign, 4 exponent bits with
 * bias 7, 3 fraction bits; no infinities, NaN = S.1111.111, largest value 448);
 * products are exact; C is fp32 if c_is_f32 != 0, else bf16 (one rounding to
 * nearest-even on store).  Layout and alignment rules of the matrix-instruction
 * kernels as for gemm_s8 (any layout, K a multiple of 128, 16-byte aligned, leading
 * dimensions multiples of 16, an m- or n-contiguous extent a multiple of 16); anything
 * else runs on the general kernel, which widens to fp32 and adds in fp32.
 * Accuracy of the sums on the matrix-instruction kernels: the 128-deep FP8 instruction
 * adds its 128 products with reduced precision - each product is aligned to the largest
 * one it is added with and cut off 13 bits below that one's leading bit - and adds the
 * result to an fp32 accumulator.  On N(0,1) operands this costs about 1e-5 relative
 * (Frobenius) against 1e-7 for a pure fp32 sum; integer-valued operands whose partial
 * sums fit 13 bits, and the general kernel, are unaffected.
 */
int gemm_f8(int transA, int transB, int64_t M, int64_t N, int64_t K,
            const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
            float beta, void *C, int64_t ldc, int c_is_f32,
            void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same for the other 8-bit float, OCP E5M2 (1 sign, 5 exponent bits with bias 15, 2
 * fraction bits; exponent 31 holds the infinities and NaN as in binary16, whose top byte
 * an E5M2 pattern is; largest finite value 57344).  Section 5(c): one more packed type
 * through the same kernels - the matrix instruction takes the format as a field.  All
 * arguments, layout rules and the accuracy note as for gemm_f8.
 */
int gemm_bf8(int transA, int transB, int64_t M, int64_t N, int64_t K,
             const uint8_t *A, int64_t lda, const uint8_t *B, int64_t ldb,
             float beta, void *C, int64_t ldc, int c_is_f32,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * int8 GEMM with exact int32 accumulation (Section 2.2 names INT8 among the packed
 * types; Section 5(c)):  C[M,N] = (accumulate ? C : 0) + A[M,K] x B[K,N].
 * A, B: device, signed 8-bit; C: device, int32; lda/ldb/ldc in elements.  Sums wrap
 * modulo 2^32 like any int32 arithmetic (|sum| < 2^31 needs K <= 131071 in the worst
 * case).  The matrix-instruction kernels take all four layouts, with K a multiple of
 * 128, 16-byte aligned bases, leading dimensions that are multiples of 16, and - for an
 * operand that is contiguous in m or n (transA == 1, transB == 0) - that extent a
 * multiple of 16; every other size or alignment runs on a plain integer kernel with
 * identical results.
 */
int gemm_s8(int transA, int transB, int64_t M, int64_t N, int64_t K,
            const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
            int accumulate, int32_t *C, int64_t ldc, void *stream);

/*
 * bf16 batch-reduce GEMM into an fp32 C (Algorithm 1 as a whole; Section 2.1:
 * the source tiles need not be contiguous).  Tile i of A starts at element
 * A_base + A_off[i], tile i of B at B_base + B_off[i]; M, N, K, lda, ldb and
 * the transpose flags are common to all tiles.  A_off and B_off are DEVICE
 * arrays of `batch` int64 element offsets (not bytes); they are read by the
 * kernel, so they must stay valid until the work has run.
 */
int brgemm_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t batch,
                const uint16_t *A_base, const int64_t *A_off, int64_t lda,
                const uint16_t *B_base, const int64_t *B_off, int64_t ldb,
                float beta, float *C, int64_t ldc,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same three operations with the fused epilogue of Section 6:
 *     C = act( beta*C + sum_i A_i x B_i + bias[n] )
 * `epilogue` is a bit set of BRGEMM_EPI_BIAS (bias: device, N fp32 values, may
 * be NULL when the flag is clear) and BRGEMM_EPI_RELU (negative results become
 * +0; NaN stays NaN).  in_dtype selects fp32, bf16 or binary16 operands; for fp32
 * operands C is fp32, for 16-bit operands C is fp32 or the operands' own type.
 * batch == 1 with NULL offset arrays is plain GEMM.
 */
int brgemm_fused(int in_dtype, int transA, int transB,
                 int64_t M, int64_t N, int64_t K, int64_t batch,
                 const void *A_base, const int64_t *A_off, int64_t lda,
                 const void *B_base, const int64_t *B_off, int64_t ldb,
                 float beta, void *C, int64_t ldc, int c_is_f32,
                 const float *bias, int epilogue,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Batched matrix multiplication (Section 5(d): "batch matmul" next to batch-reduce
 * matmul): nmat independent products of one shape in one call,
 *     C_z = beta * C_z + A_z x B_z,     z = 0 .. nmat-1   (nmat <= 65535),
 * where matrix z of an operand starts strideX ELEMENTS after matrix z-1.  strideA or
 * strideB may be 0 (all products share that operand); strideC must be at least
 * (M-1)*ldc + N so that the results do not overlap.  No reduction across z, no
 * workspace.  All other arguments as in gemm_bf16 / gemm_f32; the alignment rules
 * of the tuned kernels then also apply to the strides (multiples of 8 / 4 elements),
 * otherwise the general kernel runs.
 */
int gemm_bf16_batched(int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t nmat,
                      const uint16_t *A, int64_t lda, int64_t strideA,
                      const uint16_t *B, int64_t ldb, int64_t strideB,
                      float beta, void *C, int64_t ldc, int64_t strideC, int c_is_f32, void *stream);
int gemm_f32_batched(int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t nmat,
                     const float *A, int64_t lda, int64_t strideA,
                     const float *B, int64_t ldb, int64_t strideB,
                     float beta, float *C, int64_t ldc, int64_t strideC, void *stream);

/*
 * Pre-packed B ("VNNI-packed layout", Section 2.2 and Figure 1; the comparison of
 * packed against flat operands is the axis of the paper's evaluation, Section 6).
 * Weights that are used many times can be re-laid-out once so that the kernels
 * fetch them with straight 16-byte copies and feed the matrix instruction with
 * plain LDS reads - no transposing reads, no swizzle.
 *
 * gemm_pack_vnni_bf16: the packing of Figure 1 for any factor vnni in {2, 4, 8}:
 *     out[(k / vnni) * n_pitch * vnni + n * vnni + k % vnni] = B[k][n]
 * for a logical K x N matrix B of 16-bit elements read through transB / ldb as in
 * gemm_bf16.  out (device, 16-byte aligned) holds k_rows / vnni groups of n_pitch
 * columns of vnni elements; k_rows >= K must be a multiple of vnni, n_pitch >= N;
 * entries outside B are written as zero.  Figure 1 is vnni = 2 on a 4 x 4 matrix.
 *
 * gemm_packed_b_bytes / gemm_pack_b_bf16: the image the GEMM below reads: vnni = 8
 * (the 8 bf16 values one lane of the matrix instruction consumes), k_rows = K
 * rounded up to a multiple of 64, n_pitch = N rounded up to a multiple of 256.
 * packed: device, 16-byte aligned, at least gemm_packed_b_bytes(K, N) bytes
 * (packed_bytes says how many there are; too few is BRGEMM_INVALID_ARG).
 *
 * gemm_bf16_packed: C = act(beta*C + A x B + bias) with B given as that image
 * (packedB: device, 16-byte aligned, written by gemm_pack_b_bf16 for the same K and
 * N and complete before this call runs on the stream).  All other arguments as in
 * gemm_bf16 / brgemm_fused; results are identical to gemm_bf16 on the unpacked B up
 * to the order of the fp32 summation.
 */
int gemm_pack_vnni_bf16(int vnni, int transB, int64_t K, int64_t N, const uint16_t *B, int64_t ldb,
                        int64_t k_rows, int64_t n_pitch, uint16_t *out, void *stream);
size_t gemm_packed_b_bytes(int64_t K, int64_t N);
int gemm_pack_b_bf16(int transB, int64_t K, int64_t N, const uint16_t *B, int64_t ldb,
                     uint16_t *packed, size_t packed_bytes, void *stream);
int gemm_bf16_packed(int transA, int64_t M, int64_t N, int64_t K,
                     const uint16_t *A, int64_t lda, const uint16_t *packedB,
                     float beta, void *C, int64_t ldc, int c_is_f32,
                     const float *bias, int epilogue,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Upper bound, in bytes, of the workspace any variant may use for a problem of
 * this element type and size (batch = 1 for the GEMM calls).  Never fails;
 * returns 0 for empty problems.
 */
size_t gemm_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch);

/* Static, NUL-terminated description of a return code. */
const char *gemm_strerror(int code);

/* The hipError_t (as int) behind the calling thread's most recent
 * BRGEMM_HIP_ERROR, 0 if none. */
int gemm_last_hip_error(void);

/*
 * Tuning override, for benchmarks and tests: force the kernel variant and the
 * reduction split of subsequent calls from this thread.  variant < 0 and
 * split <= 0 restore automatic selection.  A forced variant whose alignment
 * or workspace requirements are not met makes the call fail with
 * BRGEMM_INVALID_ARG / BRGEMM_WORKSPACE_TOO_SMALL rather than silently falling back.
 * Returns BRGEMM_OK, or BRGEMM_INVALID_ARG for an unknown variant.
 */
int gemm_force_variant(int variant, int split);

/*
 * The shape -> tile table (Section 5(a): tile sizes are chosen per shape by rule): which
 * kernel variant and reduction split a plain or batch-reduce call of this element type
 * (BRGEMM_DTYPE_*), layout, size and leading dimensions would take, assuming 16-byte
 * aligned operands and `workspace_bytes` of workspace.  Pure host logic: nothing is
 * launched and no GPU is needed.  variant, split: host, receive the plan.
 */
int gemm_query_plan(int dtype, int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t batch,
                    int64_t lda, int64_t ldb, size_t workspace_bytes, int *variant, int *split);

/*
 * Tile selection by measurement (Section 5(a): the paper picks its tile sizes per target
 * by sweeping them).  gemm_tune runs C = A x B (beta = 0: C is overwritten with the
 * product) with every kernel variant and reduction split that accepts the problem, a few
 * launches each on `stream`, times them with HIP events and remembers the fastest for
 * this element type (BRGEMM_DTYPE_*), layout, M, N, K, lda, ldb and output type in a
 * table of the process; every later gemm_f32 / gemm_bf16 / gemm_f16 / brgemm_fused call
 * with batch == 1 and the same key takes that plan instead of the rule table's (if its
 * operands meet the plan's alignment rules and its workspace is large enough).
 * Unlike every other entry point this one WAITS for the device (it synchronises on its
 * own events, dozens of times) and creates and destroys two events; call it at set-up
 * time, never under graph capture.  Arguments as in gemm_bf16; variant, split (host,
 * required) and microseconds (host, may be NULL) receive the winner and its time per
 * launch.  Returns BRGEMM_OK, BRGEMM_INVALID_ARG (also for empty problems) or
 * BRGEMM_HIP_ERROR.  gemm_tune_reset forgets every remembered plan.
 */
int gemm_tune(int dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
              const void *A, int64_t lda, const void *B, int64_t ldb,
              void *C, int64_t ldc, int c_is_f32,
              void *workspace, size_t workspace_bytes, void *stream,
              int *variant, int *split, float *microseconds);
void gemm_tune_reset(void);

/* Name of variant number v ("" past the end): lets a harness enumerate them. */
const char *gemm_variant_name(int v);

/* The variant and split the calling thread's most recent successful call used. */
int gemm_last_variant(void);
int gemm_last_split(void);

/*
 * Measurement aid: the matrix-instruction rate of the device with no memory
 * traffic, i.e. the ceiling of the multiply-accumulate step of Algorithm 1 (the
 * hot loop) under the chip's own clock and power management.  Launches `blocks`
 * workgroups of 8 wavefronts (two per SIMD, as the tuned kernels run); every
 * wavefront issues `iters` x 8 independent 32x32 matrix instructions
 * (bf16: 32x32x16, fp32: 32x32x2) on operands held in registers.
 * operands: device, 6 x 64 lane values - 16 bytes (8 bf16) per lane for bf16,
 * 4 bytes per lane for fp32; the first four blocks of 64 are A fragments, the
 * last two B fragments.  Their values matter: the rate depends on them.
 * sink: device, blocks * 512 floats, receives each lane's accumulator sum.
 * flops (host, may be NULL): receives the number of floating-point operations
 * of the launch.  Returns BRGEMM_OK, BRGEMM_INVALID_ARG or BRGEMM_HIP_ERROR.
 * dtype BRGEMM_PROBE_S8 / BRGEMM_PROBE_F8 (the one-byte operand types of Section
 * 5(c)): `iters` x 32 independent 16x16 instructions per wavefront (int8: 16x16x64,
 * FP8 E4M3: 16x16x128) on 12 x 64 lane values of 16 (int8) or 32 (FP8) bytes, the
 * first eight blocks of 64 A fragments, the last four B fragments; `flops` then
 * counts integer or FP8 multiply-add operations the same way.
 * dtype BRGEMM_PROBE_BF16_16X16X32: bf16 with the instruction and register shape of
 * the 256 x 256 and the streaming kernels, `iters` x 32 independent 16x16x32
 * instructions per wavefront on 12 x 64 lane values of 16 bytes (8 bf16), the first
 * eight blocks of 64 A fragments, the last four B fragments.  This is the ceiling to
 * hold those kernels against; BRGEMM_DTYPE_BF16 (32x32x16) is the one for the 4-wave
 * 128 x 128 kernel.
 */
#define BRGEMM_PROBE_S8 3
#define BRGEMM_PROBE_F8 4
#define BRGEMM_PROBE_BF16_16X16X32 5
int gemm_mfma_probe(int dtype, const void *operands, int64_t iters, int blocks, float *sink,
                    double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BRGEMM_H */
