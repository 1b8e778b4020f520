// Register-only MFMA issue loop: the matrix-pipe rate of this chip under its own
// clock and power management, with the operand values the caller supplies and no
// LDS or memory traffic in the loop.  A measurement aid for the roofline of the
// hot loop of Algorithm 1; not part of the product path.
#include "../../include/brgemm.h"
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 pbf16x8;
typedef __attribute__((ext_vector_type(16))) float pf32x16;

// Register shape of one wave of the 4-wave 128 x 128 kernel: 4 A fragments, 2 B
// fragments, 8 accumulators of 32x32; 8 independent v_mfma_f32_32x32x16_bf16 per
// iteration.
__global__ void __launch_bounds__(512)
probe_bf16_kernel(const uint16_t *ops, int64_t iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    pbf16x8 f[6];
#pragma unroll
    for (int q = 0; q < 6; ++q)
        f[q] = *(const pbf16x8 *)(ops + ((size_t)q * 64 + lane) * 8);
    pf32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[i][r] = 0.0f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a * 4 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[4 + a], f[b], acc[a * 4 + b], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += acc[i][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// fp32: v_mfma_f32_32x32x2_f32, one float of A and of B per lane per instruction.
__global__ void __launch_bounds__(512)
probe_f32_kernel(const float *ops, int64_t iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    float f[6];
#pragma unroll
    for (int q = 0; q < 6; ++q)
        f[q] = ops[q * 64 + lane];
    pf32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[i][r] = 0.0f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a * 4 + b] = __builtin_amdgcn_mfma_f32_32x32x2f32(f[4 + a], f[b], acc[a * 4 + b], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += acc[i][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

typedef __attribute__((ext_vector_type(4))) int pi32x4;
typedef __attribute__((ext_vector_type(8))) int pi32x8;
typedef __attribute__((ext_vector_type(4))) float pf32x4;

// Register shape of one wave of the 256 x 256 ping-pong kernel and of the streaming
// kernels: 8 A and 4 B fragments, 32 accumulators of 16x16, 32 independent
// v_mfma_f32_16x16x32_bf16 per iteration (the same flop per pipe cycle as the 32x32x16
// form; each accumulator register is read and written half as often per flop).
__global__ void __launch_bounds__(512)
probe_bf16_16x16_kernel(const uint16_t *ops, int64_t iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    pbf16x8 f[12];
#pragma unroll
    for (int q = 0; q < 12; ++q)
        f[q] = *(const pbf16x8 *)(ops + ((size_t)q * 64 + lane) * 8);
    pf32x4 acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i)
        acc[i] = pf32x4{0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b)
                acc[a * 8 + b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[8 + a], f[b], acc[a * 8 + b], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            s += acc[i][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// One-byte operands in the register shape of one wave of the 256 x 256 kernel: 8 A and 4 B
// fragments, 32 accumulators of 16x16, 32 independent MFMAs per iteration.  BYTES = 16:
// v_mfma_i32_16x16x64_i8; BYTES = 32: v_mfma_f32_16x16x128_f8f6f4 on E4M3 operands.
template <int BYTES>
__global__ void __launch_bounds__(512)
probe_byte_kernel(const uint8_t *ops, int64_t iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    pi32x4 lo[12], hi[12];
#pragma unroll
    for (int q = 0; q < 12; ++q) {
        const uint8_t *src = ops + ((size_t)q * 64 + lane) * BYTES;
        lo[q] = *(const pi32x4 *)src;
        hi[q] = BYTES == 32 ? *(const pi32x4 *)(src + 16) : lo[q];
    }
    pi32x4 acc_i[32];
    pf32x4 acc_f[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        acc_i[i] = pi32x4{0, 0, 0, 0};
        acc_f[i] = pf32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                if constexpr (BYTES == 16) {
                    acc_i[a * 8 + b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(lo[8 + a], lo[b], acc_i[a * 8 + b], 0, 0, 0);
                } else {
                    const pi32x8 fa = __builtin_shufflevector(lo[8 + a], hi[8 + a], 0, 1, 2, 3, 4, 5, 6, 7);
                    const pi32x8 fb = __builtin_shufflevector(lo[b], hi[b], 0, 1, 2, 3, 4, 5, 6, 7);
                    acc_f[a * 8 + b] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fa, fb, acc_f[a * 8 + b], 0, 0, 0, 0, 0, 0);
                }
            }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            s += BYTES == 16 ? (float)acc_i[i][r] : acc_f[i][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

extern "C" int gemm_mfma_probe(int dtype, const void *operands, int64_t iters, int blocks, float *sink,
                               double *flops, void *stream)
{
    if ((dtype != BRGEMM_DTYPE_F32 && dtype != BRGEMM_DTYPE_BF16 && dtype != BRGEMM_PROBE_S8 && dtype != BRGEMM_PROBE_F8 &&
         dtype != BRGEMM_PROBE_BF16_16X16X32) ||
        !operands || !sink || iters < 0 || blocks <= 0 || blocks > (1 << 20))
        return BRGEMM_INVALID_ARG;
    // the 16x16 forms issue 32 instructions per iteration, the 32x32 forms 8
    const bool small = dtype == BRGEMM_PROBE_S8 || dtype == BRGEMM_PROBE_F8 || dtype == BRGEMM_PROBE_BF16_16X16X32;
    const double per_mfma = dtype == BRGEMM_DTYPE_BF16 ? 2.0 * 32 * 32 * 16 : dtype == BRGEMM_DTYPE_F32 ? 2.0 * 32 * 32 * 2
                            : dtype == BRGEMM_PROBE_S8 ? 2.0 * 16 * 16 * 64
                            : dtype == BRGEMM_PROBE_F8 ? 2.0 * 16 * 16 * 128 : 2.0 * 16 * 16 * 32;
    if (flops)
        *flops = per_mfma * (small ? 32.0 : 8.0) * (double)iters * 8.0 * (double)blocks;   // MFMAs per iteration x 8 waves
    if (dtype == BRGEMM_PROBE_BF16_16X16X32)
        probe_bf16_16x16_kernel<<<dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream>>>(
            (const uint16_t *)operands, iters, sink);
    else if (dtype == BRGEMM_DTYPE_BF16)
        probe_bf16_kernel<<<dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream>>>(
            (const uint16_t *)operands, iters, sink);
    else if (dtype == BRGEMM_DTYPE_F32)
        probe_f32_kernel<<<dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream>>>(
            (const float *)operands, iters, sink);
    else if (dtype == BRGEMM_PROBE_S8)
        probe_byte_kernel<16><<<dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream>>>(
            (const uint8_t *)operands, iters, sink);
    else
        probe_byte_kernel<32><<<dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream>>>(
            (const uint8_t *)operands, iters, sink);
    return hipGetLastError() == hipSuccess ? BRGEMM_OK : BRGEMM_HIP_ERROR;
}
