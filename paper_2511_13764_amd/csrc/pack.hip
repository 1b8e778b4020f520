// VNNI packing of the B operand on the device (Section 2.2, Figure 1): K is cut into
// groups of v rows and the v elements of a column within a group become adjacent,
//     out[(k / v) * n_pitch * v + n * v + k % v] = B[k][n],
// zero outside B.  v = 8 (one MFMA lane's 8 bf16 values) is the layout the GEMM
// kernels read; other factors exist for parity with the paper's worked example.
#include "common.hpp"

namespace brg {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t pu32x4;

// One thread per (group, column): v two-byte reads, coalesced along n for a K x N
// source, then one contiguous run of v elements.
__global__ void __launch_bounds__(256)
pack_vnni_kernel(int v, int transB, int64_t K, int64_t N, const uint16_t *B, int64_t ldb, int64_t groups,
                 int64_t n_pitch, uint16_t *out)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t g = blockIdx.y;
    if (n >= n_pitch || g >= groups)
        return;
    uint16_t *dst = out + (g * n_pitch + n) * v;
    if (v == 8) {
        // k-contiguous source with whole, aligned groups: the group is one 16-byte copy
        if (transB && n < N && g * 8 + 8 <= K && (ldb & 7) == 0 && (((uintptr_t)B) & 15) == 0) {
            *(pu32x4 *)dst = *(const pu32x4 *)(B + n * ldb + g * 8);
            return;
        }
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            uint32_t lo = 0, hi = 0;
            const int64_t k = g * 8 + j;
            if (n < N && k < K)
                lo = transB ? B[n * ldb + k] : B[k * ldb + n];
            if (n < N && k + 1 < K)
                hi = transB ? B[n * ldb + k + 1] : B[(k + 1) * ldb + n];
            w[j / 2] = lo | (hi << 16);
        }
        *(pu32x4 *)dst = pu32x4{w[0], w[1], w[2], w[3]};       // 16-byte aligned: v * 2 = 16
        return;
    }
    for (int j = 0; j < v; ++j) {
        const int64_t k = g * v + j;
        uint16_t e = 0;
        if (n < N && k < K)
            e = transB ? B[n * ldb + k] : B[k * ldb + n];
        dst[j] = e;
    }
}

}  // namespace

hipError_t launch_pack_vnni(int v, int transB, int64_t K, int64_t N, const uint16_t *B, int64_t ldb,
                            int64_t k_rows, int64_t n_pitch, uint16_t *out, hipStream_t stream)
{
    const int64_t groups = k_rows / v;
    if (groups == 0 || n_pitch == 0)
        return hipSuccess;
    // grid.y is limited to 65535 groups per launch
    for (int64_t g0 = 0; g0 < groups; g0 += 65535) {
        const int64_t gcount = groups - g0 < 65535 ? groups - g0 : 65535;
        const dim3 grid((unsigned)((n_pitch + 255) / 256), (unsigned)gcount);
        const int64_t k0 = g0 * v;
        const uint16_t *src = transB ? B + k0 : B + k0 * ldb;
        hipLaunchKernelGGL(pack_vnni_kernel, grid, dim3(256), 0, stream, v, transB, K > k0 ? K - k0 : 0, N, src, ldb,
                           gcount, n_pitch, out + g0 * n_pitch * v);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

}  // namespace brg
