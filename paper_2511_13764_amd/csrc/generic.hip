// General BRGEMM kernel for gfx950: any M, N, K, batch, leading dimensions,
// alignment and transpose flags.  It is the slow-but-always-correct member of
// the family; the tuned kernels take over when their alignment rules hold.
//
// Structure (Algorithm 1 of the paper, mapped to a GPU): one workgroup owns a
// 64 x 64 sub-block of C; its four wavefronts each keep a 32 x 32 accumulator
// tile in registers over the whole batch and K loops (Section 2.1, advantage
// (1)), feed it with the fp32 MFMA v_mfma_f32_32x32x2_f32, and apply beta /
// bias / ReLU / narrowing once at the end.  bf16 inputs are widened exactly to
// fp32 when they are staged into LDS, so each product is exact in fp32 and the
// sum is fp32 (the appendix listings: widen, multiply, add in f32).
#include "bf16_tiles.hpp"

namespace brg {

typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int GT = 64;      // tile edge (M and N)
constexpr int GK = 16;      // k-block
constexpr int GPAD = 1;     // LDS row padding (floats)

// KIND: 0 fp32, 1 bf16, 2 binary16, 3 FP8 E4M3, 4 FP8 E5M2
template <int KIND>
__device__ __forceinline__ float load_in(const void *p, int64_t idx)
{
    if (KIND == 1)
        return bf16_to_f32(((const uint16_t *)p)[idx]);
    if (KIND == 2)
        return f16_to_f32(((const uint16_t *)p)[idx]);
    if (KIND == 3)
        return f8e4m3_to_f32(((const uint8_t *)p)[idx]);
    if (KIND == 4)
        return f8e5m2_to_f32(((const uint8_t *)p)[idx]);
    return ((const float *)p)[idx];
}

template <int KIND>
__global__ void __launch_bounds__(256)
generic_kernel(int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t batch,
               const void *A, const int64_t *A_off, int64_t lda,
               const void *B, const int64_t *B_off, int64_t ldb,
               Epilogue epi, int split, float *partial)
{
    __shared__ float As[GK][GT + GPAD];     // [k][m]
    __shared__ float Bs[GK][GT + GPAD];     // [k][n]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.y * GT;
    const int64_t n0 = (int64_t)blockIdx.x * GT;

    // Flattened iteration space: it = i * kblocks + kb, cut into `split` ranges.
    const int64_t kblocks = (K + GK - 1) / GK;
    const int64_t total = batch * kblocks;
    const int64_t per = (total + split - 1) / split;
    const int64_t it_begin = (int64_t)blockIdx.z * per;
    const int64_t it_end = (it_begin + per < total) ? it_begin + per : total;

    f32x16 acc;
    for (int r = 0; r < 16; ++r)
        acc[r] = 0.0f;

    for (int64_t it = it_begin; it < it_end; ++it) {
        const int64_t i = it / kblocks;
        const int64_t k0 = (it - i * kblocks) * GK;
        const int64_t ao = A_off ? A_off[i] : 0;
        const int64_t bo = B_off ? B_off[i] : 0;

        // Stage the A block (64 x 16) and the B block (16 x 64) into LDS, zero-filled
        // outside the matrix.  Threads run along the operand's contiguous direction.
        for (int e = tid; e < GT * GK; e += 256) {
            int m, k;
            if (transA) { m = e % GT; k = e / GT; } else { k = e % GK; m = e / GK; }
            const int64_t gm = m0 + m, gk = k0 + k;
            float v = 0.0f;
            if (gm < M && gk < K)
                v = load_in<KIND>(A, ao + (transA ? gk * lda + gm : gm * lda + gk));
            As[k][m] = v;
        }
        for (int e = tid; e < GT * GK; e += 256) {
            int n, k;
            if (transB) { k = e % GK; n = e / GK; } else { n = e % GT; k = e / GT; }      // 2 (packed): k fastest
            const int64_t gn = n0 + n, gk = k0 + k;
            float v = 0.0f;
            if (gn < N && gk < K)
                v = load_in<KIND>(B, bo + (transB == 2 ? (gk >> 3) * ldb + gn * 8 + (gk & 7)
                                                       : transB ? gn * ldb + gk : gk * ldb + gn));
            Bs[k][n] = v;
        }
        __syncthreads();

        // v_mfma_f32_32x32x2_f32: lane l supplies A[row l%32][k = l/32] and
        // B[k = l/32][col l%32].
#pragma unroll
        for (int kk = 0; kk < GK; kk += 2) {
            const float a = As[kk + (lane >> 5)][wm * 32 + (lane & 31)];
            const float b = Bs[kk + (lane >> 5)][wn * 32 + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }

    // Accumulator layout of the 32x32 MFMA: register r of lane l holds
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    const int64_t n = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M && n < N) {
            if (split > 1)
                partial[((int64_t)blockIdx.z * M + m) * N + n] = acc[r];
            else
                epilogue_store(epi, acc[r], m, n);
        }
    }
}

__global__ void __launch_bounds__(256)
reduce_kernel(int64_t M, int64_t N, int split, const float *partial, Epilogue epi)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        float s = partial[e];
        for (int z = 1; z < split; ++z)
            s += partial[(int64_t)z * total + e];
        epilogue_store(epi, s, e / N, e % N);
    }
}

// The same sum, four consecutive columns per thread with 16-byte reads of the
// partial tiles (N a multiple of 4; C 16-byte aligned with ldc a multiple of 4).
// The slices are added in the order 0, 1, ..., split - 1, as in the scalar kernel.
__global__ void __launch_bounds__(256)
reduce4_kernel(int M, int quads_per_row, int split, const float *partial, Epilogue epi)
{
    const int q = (int)blockIdx.x * 256 + (int)threadIdx.x;
    const int m = (int)blockIdx.y;
    if (q >= quads_per_row)
        return;
    const int64_t N = (int64_t)quads_per_row * 4;
    const int64_t total = (int64_t)M * N;
    const float *src = partial + (int64_t)m * N + (int64_t)q * 4;
    f32x4 s = *(const f32x4 *)src;
    for (int z = 1; z < split; ++z)
        s += *(const f32x4 *)(src + (int64_t)z * total);
    store4_epilogue(epi, m, (int64_t)q * 4, 4, true, s[0], s[1], s[2], s[3]);
}

__global__ void __launch_bounds__(256)
scale_only_kernel(int64_t M, int64_t N, Epilogue epi)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256)
        epilogue_store(epi, 0.0f, e / N, e % N);
}

static Epilogue make_epilogue(const Problem &p)
{
    Epilogue e;
    e.beta = p.beta;
    e.C = p.C;
    e.ldc = p.ldc;
    e.c_f32 = p.c_f32;
    e.c_f16 = p.in_f16;
    e.c_i32 = p.in_s8;
    e.bias = p.bias;
    e.relu = p.relu;
    return e;
}

hipError_t launch_generic(const Problem &p)
{
    dim3 grid((unsigned)((p.N + GT - 1) / GT), (unsigned)((p.M + GT - 1) / GT), (unsigned)p.split);
    // A batched call runs one launch per matrix here (this is the slow general path).
    const int64_t esz = p.in_f8 ? 1 : in_16bit(p) ? 2 : 4, csz = p.c_f32 ? 4 : 2;
    for (int64_t z = 0; z < p.nmat; ++z) {
        Epilogue e = make_epilogue(p);
        e.C = (char *)p.C + z * p.ms_c * csz;
        const void *A = (const char *)p.A + z * p.ms_a * esz;
        const void *B = (const char *)p.B + z * p.ms_b * esz;
        if (p.in_bf16)
            hipLaunchKernelGGL(generic_kernel<1>, grid, dim3(256), 0, p.stream, p.transA,
                               p.b_packed ? 2 : p.transB, p.M, p.N, p.K, p.batch, A, p.A_off, p.lda, B, p.B_off,
                               p.ldb, e, p.split, p.partial);
        else if (p.in_f8 && p.f8_e5m2)
            hipLaunchKernelGGL(generic_kernel<4>, grid, dim3(256), 0, p.stream, p.transA, p.transB, p.M, p.N,
                               p.K, p.batch, A, p.A_off, p.lda, B, p.B_off, p.ldb, e, p.split, p.partial);
        else if (p.in_f8)
            hipLaunchKernelGGL(generic_kernel<3>, grid, dim3(256), 0, p.stream, p.transA, p.transB, p.M, p.N,
                               p.K, p.batch, A, p.A_off, p.lda, B, p.B_off, p.ldb, e, p.split, p.partial);
        else if (p.in_f16)
            hipLaunchKernelGGL(generic_kernel<2>, grid, dim3(256), 0, p.stream, p.transA, p.transB, p.M, p.N,
                               p.K, p.batch, A, p.A_off, p.lda, B, p.B_off, p.ldb, e, p.split, p.partial);
        else
            hipLaunchKernelGGL(generic_kernel<0>, grid, dim3(256), 0, p.stream, p.transA, p.transB, p.M, p.N,
                               p.K, p.batch, A, p.A_off, p.lda, B, p.B_off, p.ldb, e, p.split, p.partial);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess)
            return err;
    }
    return hipSuccess;
}

// int8 x int8 -> int32, one C element per thread, any layout: the int8 fallback.
__global__ void __launch_bounds__(256)
generic_s8_kernel(int transA, int transB, int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda,
                  const int8_t *B, int64_t ldb, int accumulate, int32_t *C, int64_t ldc)
{
    const int64_t n = (int64_t)blockIdx.x * 16 + (threadIdx.x & 15);
    const int64_t m = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4);
    if (m >= M || n >= N)
        return;
    int32_t s = accumulate ? C[m * ldc + n] : 0;
    for (int64_t k = 0; k < K; ++k) {
        const int32_t a = transA ? A[k * lda + m] : A[m * lda + k];
        const int32_t b = transB ? B[n * ldb + k] : B[k * ldb + n];
        s += a * b;
    }
    C[m * ldc + n] = s;
}

hipError_t launch_generic_s8(const Problem &p)
{
    if ((p.M + 15) / 16 > 65535)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)((p.N + 15) / 16), (unsigned)((p.M + 15) / 16));
    hipLaunchKernelGGL(generic_s8_kernel, grid, dim3(256), 0, p.stream, p.transA, p.transB, p.M, p.N, p.K,
                       (const int8_t *)p.A, p.lda, (const int8_t *)p.B, p.ldb, p.beta != 0.0f ? 1 : 0,
                       (int32_t *)p.C, p.ldc);
    return hipGetLastError();
}

static unsigned elementwise_grid(int64_t total)
{
    int64_t g = (total + 255) / 256;
    if (g > 256 * 16)
        g = 256 * 16;
    if (g < 1)
        g = 1;
    return (unsigned)g;
}

hipError_t launch_reduce(const Problem &p)
{
    if ((p.N & 3) == 0 && (p.ldc & 3) == 0 && (((uintptr_t)p.C) & 15) == 0 && p.M <= 65535) {
        const int quads = (int)(p.N / 4);
        hipLaunchKernelGGL(reduce4_kernel, dim3((unsigned)((quads + 255) / 256), (unsigned)p.M), dim3(256), 0,
                           p.stream, (int)p.M, quads, p.split, p.partial, make_epilogue(p));
        return hipGetLastError();
    }
    hipLaunchKernelGGL(reduce_kernel, dim3(elementwise_grid(p.M * p.N)), dim3(256), 0, p.stream, p.M, p.N,
                       p.split, p.partial, make_epilogue(p));
    return hipGetLastError();
}

hipError_t launch_scale_only(const Problem &p)
{
    for (int64_t z = 0; z < p.nmat; ++z) {
        Epilogue e = make_epilogue(p);
        e.C = (char *)p.C + z * p.ms_c * (p.c_f32 ? 4 : 2);
        hipLaunchKernelGGL(scale_only_kernel, dim3(elementwise_grid(p.M * p.N)), dim3(256), 0, p.stream, p.M, p.N, e);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess)
            return err;
    }
    return hipSuccess;
}

}  // namespace brg
