// Shared declarations of the GPU library (host dispatch <-> kernel launchers).
// Not part of the public interface; the public interface is include/brgemm.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace brg {

// One fully validated problem: C = act(beta*C + sum_i A_i x B_i + bias)
// (input/output statement of Algorithm 1; Section 6 for bias and ReLU).
struct Problem {
    int in_bf16;            // 1: A, B are bf16 bit patterns
    int in_f16;             // 1: A, B are IEEE binary16 bit patterns
    int in_s8;              // 1: A, B are signed 8-bit integers, C is int32
    int in_f8;              // 1: A, B are 8-bit floats (all four 0: fp32) ...
    int f8_e5m2;            // ... of the E5M2 kind (0: E4M3)
    int transA, transB;     // 1: stored transposed (K x M / N x K), row-major
    int64_t M, N, K, batch;
    const void *A;          // base of every A_i
    const int64_t *A_off;   // device, batch element offsets, or nullptr (all zero)
    int64_t lda;
    const void *B;
    const int64_t *B_off;
    int64_t ldb;
    // 1: B is the image written by the packer (groups of 8 k, Section 2.2 / Figure 1):
    // element (k, n) at ((k / 8) * n_pitch + n) * 8 + k % 8 with ldb = n_pitch * 8,
    // n_pitch a multiple of 256, k padded to a multiple of 64 with zeros; transB is 0.
    int b_packed;
    float beta;
    void *C;
    int64_t ldc;
    int c_f32;              // 1: C is fp32; 0: the 16-bit type of the operands (bf16 / binary16)
    const float *bias;      // nullptr or N fp32 values
    int relu;
    // Reduction split: the flattened (batch x k-block) iteration space is cut into
    // `split` contiguous ranges, one per blockIdx.z; split > 1 writes raw fp32
    // partial tiles to `partial` (split x M x N, dense) and a second kernel sums
    // them in a fixed order and applies the epilogue (deterministic).
    int split;
    float *partial;
    // Batched (non-reduce) matmul, Section 5(d): nmat independent problems of the same
    // shape; matrix z uses A + z*ms_a, B + z*ms_b, C + z*ms_c (element strides, 0 = the
    // operand is shared).  nmat > 1 excludes tile offsets and a split.
    int64_t nmat, ms_a, ms_b, ms_c;
    hipStream_t stream;
};

// fp32 -> bf16, round to nearest even, NaN -> quiet NaN (Section 4.3: one
// narrowing after the whole sum).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Two fp32 -> one register of two bf16 (first value in the low half) with the
// hardware conversion v_cvt_pk_bf16_f32 (round to nearest even, NaN stays NaN).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const bf16x2_t r = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h)
{
    return __uint_as_float((uint32_t)h << 16);
}

// binary16 (the FP16 of Section 2.2): hardware conversions, round to nearest even on
// narrowing, subnormals kept.
__device__ __forceinline__ float f16_to_f32(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}
__device__ __forceinline__ uint16_t f32_to_f16_rne(float f)
{
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi)
{
    return (uint32_t)f32_to_f16_rne(lo) | ((uint32_t)f32_to_f16_rne(hi) << 16);
}
// FP8 E4M3 (OCP: bias 7, no infinities, NaN = S.1111.111) widened exactly.
__device__ __forceinline__ float f8e4m3_to_f32(uint8_t b)
{
    const int e = (b >> 3) & 15, f = b & 7;
    float v;
    if (e == 15 && f == 7)
        v = __uint_as_float(0x7fc00000u);
    else if (e == 0)
        v = (float)f * 0.001953125f;                         // f * 2^-9
    else
        v = __uint_as_float((uint32_t)(e + 120) << 23 | (uint32_t)f << 20);     // (1 + f/8) * 2^(e-7)
    return (b & 0x80) ? -v : v;
}
// FP8 E5M2 (OCP: bias 15, infinities and NaN as in binary16, whose top byte it is).
__device__ __forceinline__ float f8e5m2_to_f32(uint8_t b)
{
    return f16_to_f32((uint16_t)((uint16_t)b << 8));
}
// 16-bit C element of either kind.
__device__ __forceinline__ float c16_to_f32(uint16_t h, int f16) { return f16 ? f16_to_f32(h) : bf16_to_f32(h); }
__device__ __forceinline__ uint32_t pack_c16x2(float lo, float hi, int f16)
{
    return f16 ? pack_f16x2(lo, hi) : pack_bf16x2(lo, hi);
}


// Epilogue parameters as the kernels see them.
struct Epilogue {
    float beta;
    void *C;
    int64_t ldc;
    int c_f32;
    int c_f16;              // with c_f32 == 0: 1 = binary16 C, 0 = bf16 C
    int c_i32;              // 1: C is int32 and the accumulators hold int32 bit patterns
                            // (int8 path; beta is 0 or 1 and means "add the old C")
    const float *bias;
    int relu;
};

// v = finished sum for element (m, n): apply beta*C_old, bias, ReLU (fp32) and
// return the value to store.  beta == 0 never reads C.
__device__ __forceinline__ float epilogue_value(const Epilogue &e, float v, int64_t m, int64_t n)
{
    if (e.beta != 0.0f) {
        float old = e.c_f32 ? ((const float *)e.C)[m * e.ldc + n]
                            : c16_to_f32(((const uint16_t *)e.C)[m * e.ldc + n], e.c_f16);
        v = fmaf(e.beta, old, v);
    }
    if (e.bias)
        v += e.bias[n];
    if (e.relu)
        v = (v < 0.0f) ? 0.0f : v;      // NaN stays NaN (fmaxf would drop it)
    return v;
}

__device__ __forceinline__ void epilogue_store(const Epilogue &e, float v, int64_t m, int64_t n)
{
    if (e.c_i32) {
        int32_t r = __float_as_int(v);
        if (e.beta != 0.0f)
            r += ((const int32_t *)e.C)[m * e.ldc + n];
        ((int32_t *)e.C)[m * e.ldc + n] = r;
        return;
    }
    v = epilogue_value(e, v, m, n);
    if (e.c_f32)
        ((float *)e.C)[m * e.ldc + n] = v;
    else
        ((uint16_t *)e.C)[m * e.ldc + n] = e.c_f16 ? f32_to_f16_rne(v) : f32_to_bf16_rne(v);
}

inline bool in_16bit(const Problem &p) { return p.in_bf16 || p.in_f16; }
// Operand kinds as template arguments of the kernels that move 128-byte k-rows.
constexpr int KIND_BF16 = 0, KIND_F16 = 1, KIND_S8 = 2, KIND_F8 = 3, KIND_BF8 = 4;      // F8: E4M3, BF8: E5M2
constexpr bool kind_is_f8(int kind) { return kind == KIND_F8 || kind == KIND_BF8; }
constexpr bool kind_is_8bit(int kind) { return kind == KIND_S8 || kind_is_f8(kind); }
inline bool in_8bit(const Problem &p) { return p.in_s8 || p.in_f8; }

// ---- launchers (each returns the hipError_t of its launch) -------------------

// General kernel: any shape, alignment, transposes, batch, split.
hipError_t launch_generic(const Problem &p);
// Sum `split` partial tiles and apply the epilogue.
hipError_t launch_reduce(const Problem &p);
// beta-only pass for K == 0 or batch == 0: C = act(beta*C + bias).
hipError_t launch_scale_only(const Problem &p);
// VNNI-v packing of a K x N matrix of 16-bit elements into k_rows / v groups of
// n_pitch columns (zero outside the matrix).
// Any-layout int8 GEMM into int32 (plain integer loop; the fallback of the int8 path).
hipError_t launch_generic_s8(const Problem &p);
hipError_t launch_pack_vnni(int v, int transB, int64_t K, int64_t N, const uint16_t *B, int64_t ldb,
                            int64_t k_rows, int64_t n_pitch, uint16_t *out, hipStream_t stream);

}  // namespace brg
