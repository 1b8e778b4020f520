// Tuned fp32 GEMM kernel for gfx950: 128 x 128 x 32 workgroup tile, 8 wavefronts,
// each keeping a 64 x 32 accumulator tile (two v_mfma_f32_32x32x2_f32 tiles, 32
// registers) in registers for the whole K loop - the fp32 branch of Algorithm 1
// (broadcast a column of A, load a chunk of B, fused multiply-add into the resident
// accumulators), with the matrix instruction in the role of vector.fma.
//
// fp32 MFMA runs at 1/16 of the bf16 rate, so per k-block the 64 MFMAs of a SIMD
// take ~4096 cycles against 32 KiB of loads and ~100 KiB of LDS reads per CU: the
// kernel is bound by the matrix pipe; two waves per SIMD cover each other's load
// issue and LDS latency, and a three-stage LDS ring with its one barrier per block in
// mid-block gives every load a whole k-block of time to land.  Global -> LDS copies
// use the scalar-base form of global_load_lds_dwordx4, threaded between the MFMAs.
//
// LDS images.  An operand whose contiguous direction is k keeps 128-byte rows with
// the 16-byte chunk c of row r at position c ^ ((r >> 1) & 7) (same image as the
// bf16 kernels); a lane fetches 4 consecutive k with one 128-bit read and feeds them
// to 4 successive MFMAs.  The k order inside the MFMA is free as long as both
// operands agree: MFMA (j, t) contracts k = 8j + t (lanes 0-31) and 8j + 4 + t
// (lanes 32-63).  An operand whose contiguous direction is m or n keeps 512-byte
// k-rows; the lane needs one element per MFMA (32-bit read), and the chunk position
// is c ^ 8 for k-rows with bit 2 set so that the two half-waves hit different banks.
#include "bf16_tiles.hpp"

namespace brg {

namespace {

constexpr int FB = 128;                 // tile edge (M and N)
constexpr int FK = 32;                  // k-block (floats) = 128 bytes
constexpr uint32_t F_OP_BYTES = FB * FK * 4;        // 16 KiB per operand per stage
constexpr uint32_t F_STAGE = 2 * F_OP_BYTES;

struct F32Args {
    int64_t M, N, K;
    const float *A;
    int64_t lda;
    const float *B;
    int64_t ldb;
    Epilogue epi;
    int split;
    float *partial;
    int tiles_m, tiles_n;
    int64_t ms_a, ms_b, ms_c;       // element strides between the matrices of a batched call
};

// k-contiguous operand: reuse the 128-byte-row image of the bf16 tiles (a float row
// of 32 k is byte-identical to a bf16 row of 64 k); leading dimensions are passed in
// 2-byte units.
typedef KMajorTile<FB, 4> FKTile;

// m/n-contiguous operand: 32 k-rows of 128 floats.
struct FMNTile {
    __device__ static int64_t instr_stride_bytes(int64_t ld) { return 2 * ld * 4; }
    // variant = (g >> 1) & 1 of wave-load g (k-row bit 2)
    __device__ static uint32_t lane_off_bytes(int variant, int lane, int64_t ld)
    {
        const int c = (lane & 31) ^ (variant << 3);
        return (uint32_t)((int64_t)(lane >> 5) * ld * 4 + 16 * c);
    }
    __device__ static bool lane_valid(int g, int lane, int64_t col0, int64_t col_limit)
    {
        const int c = (lane & 31) ^ (((g >> 1) & 1) << 3);
        return col0 + 4 * c < col_limit;
    }
    // element k = 8j + 4*(lane/32) + t of column col_base + t32*32 + lane%32
    __device__ static float read(LDS_AS char *tile, int col_base, int t32, int j, int t, int lane)
    {
        const int h = lane >> 5;
        const int k = 8 * j + 4 * h + t;
        const int col = col_base + t32 * 32 + (lane & 31);
        const int c = (col >> 2) ^ (h << 3);
        return *(LDS_AS float *)(tile + k * 512 + (c << 4) + (col & 3) * 4);
    }
};

}  // namespace

// NW = 8: two waves per SIMD (wave tile 64 x 32), which hides each wave's load issue
// and LDS latency behind the other's MFMAs; NW = 4: one wave per SIMD (wave tile 64 x 64).
template <bool A_KMAJ, bool B_KMAJ, int NW>
__global__ void __launch_bounds__(NW * 64)
f32_mfma_kernel(F32Args p)
{
    constexpr int WNW = NW / 2;             // waves along N
    constexpr int WN = FB / WNW;            // wave tile width: 64 or 32
    constexpr int TN = WN / 32;             // 32-column MFMA tiles per wave
    constexpr int PER_OP = 16 / NW;         // wave-loads per wave per operand per block

    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    LDS_AS char *smem = (LDS_AS char *)smem_generic;
    p.A += (int64_t)blockIdx.z * p.ms_a;
    p.B += (int64_t)blockIdx.z * p.ms_b;
    p.epi.C = (float *)p.epi.C + (int64_t)blockIdx.z * p.ms_c;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / WNW, wn = w % WNW;

    int tm, tn;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * FB, n0 = (int64_t)tn * FB;

    const int kblocks = (int)(p.K / FK);
    const int per = (kblocks + p.split - 1) / p.split;
    const int it_begin = (int)blockIdx.y * per;
    const int it_end = (it_begin + per < kblocks) ? it_begin + per : kblocks;
    const int n_iter = it_end - it_begin;

    // Global -> LDS addressing: scalar base + wave-load index * stride + lane offset.
    const int64_t a_stride = A_KMAJ ? FKTile::instr_stride_bytes(2 * p.lda) : FMNTile::instr_stride_bytes(p.lda);
    const int64_t b_stride = B_KMAJ ? FKTile::instr_stride_bytes(2 * p.ldb) : FMNTile::instr_stride_bytes(p.ldb);
    const uint32_t a_off0 = A_KMAJ ? FKTile::lane_off_bytes(0, lane, 2 * p.lda) : FMNTile::lane_off_bytes(0, lane, p.lda);
    const uint32_t a_off1 = A_KMAJ ? FKTile::lane_off_bytes(1, lane, 2 * p.lda) : FMNTile::lane_off_bytes(1, lane, p.lda);
    const uint32_t b_off0 = B_KMAJ ? FKTile::lane_off_bytes(0, lane, 2 * p.ldb) : FMNTile::lane_off_bytes(0, lane, p.ldb);
    const uint32_t b_off1 = B_KMAJ ? FKTile::lane_off_bytes(1, lane, 2 * p.ldb) : FMNTile::lane_off_bytes(1, lane, p.ldb);
    const int64_t a_kstep = A_KMAJ ? (int64_t)FK : (int64_t)FK * p.lda;      // floats per k-block
    const int64_t b_kstep = B_KMAJ ? (int64_t)FK : (int64_t)FK * p.ldb;
    const float *ld_a = p.A + (A_KMAJ ? m0 * p.lda : m0) + (int64_t)it_begin * a_kstep;
    const float *ld_b = p.B + (B_KMAJ ? n0 * p.ldb : n0) + (int64_t)it_begin * b_kstep;

    // Wave-load q (0..2*PER_OP-1) of this wave for the block at ld_a / ld_b: A first, then B.
    auto issue_one = [&](int stage, int q) {
        const bool is_a = q < PER_OP;
        const int g = w * PER_OP + (q % PER_OP);
        const char *base = is_a ? (const char *)ld_a + (int64_t)g * a_stride : (const char *)ld_b + (int64_t)g * b_stride;
        bool variant, on;
        if (is_a) {
            variant = A_KMAJ ? (g & 1) : ((g >> 1) & 1);
            on = A_KMAJ ? FKTile::lane_valid(g, lane, m0, p.M) : FMNTile::lane_valid(g, lane, m0, p.M);
        } else {
            variant = B_KMAJ ? (g & 1) : ((g >> 1) & 1);
            on = B_KMAJ ? FKTile::lane_valid(g, lane, n0, p.N) : FMNTile::lane_valid(g, lane, n0, p.N);
        }
        const uint32_t off = is_a ? (variant ? a_off1 : a_off0) : (variant ? b_off1 : b_off0);
        const uint32_t dst = (uint32_t)stage * F_STAGE + (is_a ? 0u : F_OP_BYTES) + (uint32_t)g * 1024u;
        if (on)
            load16_to_lds_saddr(base, off, (uint32_t)(size_t)(smem + dst));
    };
    auto advance = [&]() { ld_a += a_kstep; ld_b += b_kstep; };

    f32x16 acc[TN][2];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[a][b][r] = 0.0f;

    // Fragments of one j-step (8 k): per 32-row MFMA tile 4 floats per lane.
    f32x4 fa[2][2], fb[2][TN];         // [buffer][tile]
    auto read_step = [&](int stage, int j, int buf) {
        LDS_AS char *at = smem + (uint32_t)stage * F_STAGE;
        LDS_AS char *bt = at + F_OP_BYTES;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (A_KMAJ) {
                fa[buf][t] = *(LDS_AS f32x4 *)(at + FKTile::frag_byte(wm * 64, t, j, lane));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    fa[buf][t][e] = FMNTile::read(at, wm * 64, t, j, e, lane);
            }
        }
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            if (B_KMAJ) {
                fb[buf][t] = *(LDS_AS f32x4 *)(bt + FKTile::frag_byte(wn * WN, t, j, lane));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    fb[buf][t][e] = FMNTile::read(bt, wn * WN, t, j, e, lane);
            }
        }
    };
    // The same reads one at a time (unit u: the A tiles first, then the B tiles), so
    // that they can be placed between individual MFMAs.
    // (An m/n-contiguous operand is read two consecutive k at a time: the two 32-bit reads sit
    // 512 bytes apart and become one ds_read2st64_b32, which halves the LDS instructions of that
    // operand - they, not the bytes, are what the matrix pipe loses time to.)
    constexpr int UA = A_KMAJ ? 2 : 4, UB = B_KMAJ ? TN : 2 * TN, UNITS = UA + UB;
    auto read_unit = [&](int stage, int j, int buf, auto uc) {
        constexpr int u = decltype(uc)::value;
        LDS_AS char *at = smem + (uint32_t)stage * F_STAGE;
        LDS_AS char *bt = at + F_OP_BYTES;
        if constexpr (u < UA) {
            if constexpr (A_KMAJ) {
                fa[buf][u] = *(LDS_AS f32x4 *)(at + FKTile::frag_byte(wm * 64, u, j, lane));
            } else {
                fa[buf][u / 2][2 * (u % 2)] = FMNTile::read(at, wm * 64, u / 2, j, 2 * (u % 2), lane);
                fa[buf][u / 2][2 * (u % 2) + 1] = FMNTile::read(at, wm * 64, u / 2, j, 2 * (u % 2) + 1, lane);
            }
        } else {
            constexpr int v = u - UA;
            if constexpr (B_KMAJ) {
                fb[buf][v] = *(LDS_AS f32x4 *)(bt + FKTile::frag_byte(wn * WN, v, j, lane));
            } else {
                fb[buf][v / 2][2 * (v % 2)] = FMNTile::read(bt, wn * WN, v / 2, j, 2 * (v % 2), lane);
                fb[buf][v / 2][2 * (v % 2) + 1] = FMNTile::read(bt, wn * WN, v / 2, j, 2 * (v % 2) + 1, lane);
            }
        }
    };
    // One j-step: 8 * TN MFMAs with this wave's other work threaded between them.  An
    // MFMA holds the pipe for 64 cycles after it issues, so whatever the wave issues
    // right behind it is free; done in a clump after the last MFMA it would leave the
    // pipe idle (the other wave of the SIMD runs the same code at the same time).  After
    // MFMA 0: a quarter of the loads for block it + 2; after MFMAs 1..: the fragment reads
    // of step j + 1, spread evenly.  Operands swapped (B first): the 32x32 result is C^T,
    // so a lane owns row m = lane%32 and 4 consecutive columns per group of 4 registers.
    constexpr int NM = 8 * TN;
    constexpr int L = 2 * PER_OP;               // loads per wave per block
    auto step = [&](int cur, int nxt, auto jc, bool has_next, bool more, int fill) {
        constexpr int j = decltype(jc)::value;
        constexpr int buf = j & 1;
        static_for<0, NM>([&](auto ic) {
            constexpr int idx = decltype(ic)::value;
            constexpr int e = idx / (2 * TN), a = (idx / 2) % TN, b = idx % 2;
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[buf][a][e], fa[buf][b][e], acc[a][b], 0, 0, 0);
            if constexpr (j >= 2 && (idx == 0 || idx == NM / 2)) {
                // second half of the block: the loads of block it + 2, L / 4 at a time
                if (more) {
#pragma unroll
                    for (int q = 0; q < L / 4; ++q)
                        issue_one(fill, ((j - 2) * 2 + (idx == 0 ? 0 : 1)) * (L / 4) + q);
                }
            }
            if constexpr (idx > 0) {
                // the fragment reads of the next step (of the next block after step 3)
                static_for<0, UNITS>([&](auto uc) {
                    if constexpr (1 + decltype(uc)::value * (NM - 1) / UNITS == idx) {
                        if constexpr (j < 3)
                            read_unit(cur, j + 1, buf ^ 1, uc);
                        else if (has_next)
                            read_unit(nxt, 0, buf ^ 1, uc);
                    }
                });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // Three LDS stages and one barrier per k-block, placed in the MIDDLE of the block:
    // after the first two of its four 8-deep steps a wave waits for its loads of block
    // it + 1 (requested during the second half of block it - 1, a whole block of time
    // ago, and the only loads outstanding at that point - so the wait is a plain
    // vmcnt(0) and needs no counting) and the barrier publishes block it + 1 and proves
    // block it - 1 fully read.  The second half of block `it` requests block it + 2 into
    // the slot of block it - 1 and, under its last MFMAs, already reads the first
    // fragments of block it + 1: neither LDS latency nor a barrier sits between the last
    // MFMA of one block and the first of the next.
    if (n_iter > 0) {
#pragma unroll
        for (int q = 0; q < L; ++q)
            issue_one(0, q);
        advance();
        if (n_iter > 1) {
#pragma unroll
            for (int q = 0; q < L; ++q)
                issue_one(1, q);
            advance();
        }
        wait_vmcnt0();
        block_sync();
        read_step(0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);

        int cur = 0;
        for (int it = 0; it < n_iter; ++it) {
            const int nxt = cur == 2 ? 0 : cur + 1;
            const int fill = cur == 0 ? 2 : cur - 1;        // slot of block it - 1 = slot of block it + 2
            const bool more = it + 2 < n_iter;
            const bool has_next = it + 1 < n_iter;
            step(cur, nxt, std::integral_constant<int, 0>{}, has_next, more, fill);
            step(cur, nxt, std::integral_constant<int, 1>{}, has_next, more, fill);
            wait_vmcnt0();                      // block it + 1 (nothing younger is in flight here)
            block_sync();
            step(cur, nxt, std::integral_constant<int, 2>{}, has_next, more, fill);
            step(cur, nxt, std::integral_constant<int, 3>{}, has_next, more, fill);
            if (more)
                advance();
            cur = nxt;
        }
        wait_lgkmcnt0();
        block_sync();                           // every wave is done with the LDS stages
    }

    // ---- epilogue: beta*C, bias, ReLU, store (or raw partial tile for a split).
    // A lane holds 4 consecutive columns of 32 different rows, which would make every
    // global access touch 32 cache lines for 32 bytes each.  Each 32x32 accumulator
    // block therefore goes through this wave's own 4.5 KiB of LDS (all stages are free
    // after the last barrier; 144-byte row pitch: conflict-free 128-bit writes) and is
    // read back row-wise, so that one instruction covers 8 rows x 128 bytes: whole
    // cache lines for the store and for the read of the old C when beta != 0.
    constexpr int EPI_LD = 36;
    LDS_AS float *stage = (LDS_AS float *)(smem + (uint32_t)w * (32 * EPI_LD * 4));
    const bool to_partial = p.split > 1;
    float *part = to_partial ? p.partial + (int64_t)blockIdx.y * p.M * p.N : nullptr;
    const bool vec = to_partial ? ((p.N & 3) == 0) : ((p.epi.ldc & 3) == 0 && (((uintptr_t)p.epi.C) & 15) == 0);
    static_for<0, 2 * TN>([&](auto bc) {
        constexpr int b = decltype(bc)::value / TN, a = decltype(bc)::value % TN;
        asm volatile("" ::: "memory");
        static_for<0, 4>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            *(LDS_AS f32x4 *)(stage + (lane & 31) * EPI_LD + 8 * q + 4 * (lane >> 5)) =
                f32x4{acc[a][b][4 * q + 0], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
        });
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = i * 64 + lane;
            const int row = idx >> 3, c4 = idx & 7;
            const f32x4 v = *(LDS_AS f32x4 *)(stage + row * EPI_LD + c4 * 4);
            const int64_t m = m0 + wm * 64 + b * 32 + row;
            const int64_t n = n0 + wn * WN + a * 32 + c4 * 4;
            if (m < p.M) {
                if (to_partial)
                    store4_partial(part + m * p.N + n, p.N - n, vec, v[0], v[1], v[2], v[3]);
                else
                    store4_epilogue(p.epi, m, n, p.N - n, vec, v[0], v[1], v[2], v[3]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    });
}

hipError_t launch_f32_128x128(const Problem &p)
{
    F32Args a;
    a.M = p.M; a.N = p.N; a.K = p.K;
    a.A = (const float *)p.A; a.lda = p.lda;
    a.B = (const float *)p.B; a.ldb = p.ldb;
    a.epi.beta = p.beta; a.epi.C = p.C; a.epi.ldc = p.ldc; a.epi.c_f32 = 1; a.epi.c_f16 = 0; a.epi.c_i32 = 0;
    a.epi.bias = p.bias; a.epi.relu = p.relu;
    a.split = p.split; a.partial = p.partial;
    a.ms_a = p.ms_a; a.ms_b = p.ms_b; a.ms_c = p.ms_c;
    a.tiles_m = (int)((p.M + FB - 1) / FB);
    a.tiles_n = (int)((p.N + FB - 1) / FB);
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)p.split, (unsigned)p.nmat);
    const size_t lds = 3 * (size_t)F_STAGE;
    const bool ak = p.transA == 0, bk = p.transB == 1;
    void (*kern)(F32Args) = nullptr;
    constexpr int NW = 8;
    if (ak && bk) kern = f32_mfma_kernel<true, true, NW>;
    else if (ak && !bk) kern = f32_mfma_kernel<true, false, NW>;
    else if (!ak && bk) kern = f32_mfma_kernel<false, true, NW>;
    else kern = f32_mfma_kernel<false, false, NW>;
    static thread_local const void *configured[4] = {nullptr};
    bool done = false;
    for (const void *c : configured)
        done = done || c == (const void *)kern;
    if (!done) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        for (auto &c : configured)
            if (!c) { c = (const void *)kern; break; }
    }
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), lds, p.stream, a);
    return hipGetLastError();
}

// fp32 operands, plain GEMM (no tile offsets), K a multiple of 32, 16-byte aligned
// bases, leading dimensions multiples of 4, and an m/n-contiguous operand must have
// its extent a multiple of 4 (whole 16-byte chunks).
bool f32_mfma_eligible(const Problem &p)
{
    if (in_16bit(p) || in_8bit(p) || !p.c_f32 || p.A_off || p.batch != 1)
        return false;
    if (p.K % FK != 0)
        return false;
    if (((uintptr_t)p.A & 15) || ((uintptr_t)p.B & 15) || (p.lda & 3) || (p.ldb & 3))
        return false;
    if ((p.ms_a & 3) || (p.ms_b & 3))
        return false;
    if (p.transA == 1 && (p.M & 3))
        return false;
    if (p.transB == 0 && (p.N & 3))
        return false;
    if (p.lda >= (1 << 21) || p.ldb >= (1 << 21) || p.M * p.N >= ((int64_t)1 << 40))
        return false;
    return true;
}

}  // namespace brg
