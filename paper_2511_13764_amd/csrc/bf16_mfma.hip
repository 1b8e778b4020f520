// Tuned bf16 BRGEMM kernel for gfx950 (MI355X) with 4 wavefronts: bf16 operands, fp32
// accumulation, 128 x 128 x 64 workgroup tile (small and medium grids, batch-reduce).
//
// Mapping of the paper's scheme (Algorithm 1; Sections 2.3 and 3.1) to CDNA4:
//   microkernel  = one workgroup (4 wavefronts) owning a BM x BN block of C,
//                  fed from LDS in 64-deep k-blocks;
//   nanokernel   = one wavefront's (BM/2) x (BN/2) register tile, built from
//                  v_mfma_f32_32x32x16_bf16 and kept in registers for the whole
//                  batch and K loops (no spills: a 64 x 64 wave tile takes 64
//                  accumulator registers per lane).  This latency-bound kernel keeps
//                  the 32x32x16 form: with one wave per SIMD the four 16-deep slices
//                  give a finer interleave of LDS reads and MFMAs than the 16x16x32
//                  form, which measured 10-15 % slower here (it wins only where the
//                  chip is power-limited, in the 8-wave kernel).
//   "Flat" operands (Section 4.3): an operand whose contiguous direction is k
//   feeds the matrix instruction with plain 128-bit LDS reads; one whose
//   contiguous direction is m or n is re-laid-out on the way out of LDS with the
//   transposing read ds_read_b64_tr_b16, overlapped with the MFMAs - the role the
//   software-pipelined vpunpck packing plays in the paper's AMX kernels.
//
// Data movement: global -> LDS goes through global_load_lds_dwordx4 (16 bytes per
// lane, no register staging).  One wave instruction fills 1 KiB of LDS in lane
// order, so the swizzle that keeps the LDS reads bank-conflict free is applied by
// choosing WHICH 16 global bytes each lane fetches.  Two LDS stages; the block
// for k-step t+2 is requested while block t's last slice is being multiplied.
#include "bf16_tiles.hpp"

namespace brg {

template <int BM, int BN, bool A_KMAJ, int B_LAY, int KIND>
__global__ void __launch_bounds__(256)
bf16_mfma_kernel(Bf16Args p)
{
    typedef typename TileOf<BM, 4, A_KMAJ ? LAY_K : LAY_MN, KIND>::type ATile;
    typedef typename TileOf<BN, 4, B_LAY, KIND>::type BTile;
    constexpr int WM = BM / 2, WN = BN / 2;         // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;       // MFMA tiles per wave tile
    constexpr uint32_t A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr uint32_t STAGE = A_BYTES + B_BYTES;

    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    LDS_AS char *smem = (LDS_AS char *)smem_generic;
    select_matrix(p);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;

    int tm, tn;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    // Reduction range of this workgroup: flattened (batch, k-block) iterations
    // (the host guarantees batch * K/64 < 2^31).
    const int kblocks = (int)(p.K / BK);
    const int total = (int)p.batch * kblocks;
    const int per = (total + p.split - 1) / p.split;
    const int it_begin = (int)blockIdx.y * per;
    const int it_end = (it_begin + per < total) ? it_begin + per : total;
    const int n_iter = it_end - it_begin;

    // Per-lane source offsets (bytes from the block origin), fixed for the whole kernel;
    // the block origin is a wave-uniform pointer (scalar-base form of the loads).
    uint32_t a_src[ATile::kPerWave], b_src[BTile::kPerWave];
#pragma unroll
    for (int j = 0; j < ATile::kPerWave; ++j)
        a_src[j] = ATile::src_rel_bytes(w, j, lane, m0, p.M, p.lda);
#pragma unroll
    for (int j = 0; j < BTile::kPerWave; ++j)
        b_src[j] = BTile::src_rel_bytes(w, j, lane, n0, p.N, p.ldb);
    const int64_t a_origin = ATile::origin(m0, p.lda);
    const int64_t b_origin = BTile::origin(n0, p.ldb);
    const int64_t a_kstep = ATile::kstep(p.lda);
    const int64_t b_kstep = BTile::kstep(p.ldb);

    // Load cursor: the (batch index, k-block) of the next block to request, and the
    // operand pointers that go with it.  Advanced without divisions.
    int ld_i = n_iter > 0 ? it_begin / kblocks : 0;
    int ld_kb = n_iter > 0 ? it_begin - ld_i * kblocks : 0;
    TileOffsets offs_a, offs_b;                 // this wave's window of the tile offsets
    if (p.A_off) {
        offs_a.init(p.A_off, p.batch, ld_i, lane);
        offs_b.init(p.B_off, p.batch, ld_i, lane);
    }
    const uint16_t *ld_a = uniform_ptr(p.A + (p.A_off ? offs_a.get(ld_i, lane) : 0) + a_origin + ld_kb * a_kstep);
    const uint16_t *ld_b = uniform_ptr(p.B + (p.B_off ? offs_b.get(ld_i, lane) : 0) + b_origin + ld_kb * b_kstep);
    // Tile offsets live in device memory, so their alignment cannot be checked on the
    // host: if any A_off / B_off is not a multiple of 8 elements (16 bytes) the whole
    // workgroup stages its blocks through registers with 2-byte loads instead.
    bool direct = true;
    if (p.A_off) {
        int ok = 1;
        for (int i = tid; i < (int)p.batch; i += 256)
            ok &= (((p.A_off[i] | p.B_off[i]) & 7) == 0);
        direct = __syncthreads_and(ok) != 0;
    }
    auto staged16 = [&](const char *gc, uint32_t lds_byte) {
        const uint16_t *g = (const uint16_t *)gc;
        s16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = (short)g[e];
        *(LDS_AS s16x8 *)(smem + lds_byte + lane * 16) = v;
    };
    auto issue_loads = [&](int stage) {
        const uint32_t base = (uint32_t)stage * STAGE;
        const char *ga = (const char *)ld_a, *gb = (const char *)ld_b;
        if (direct) {
#pragma unroll
            for (int j = 0; j < ATile::kPerWave; ++j)
                load16_to_lds_saddr(ga, a_src[j], (uint32_t)(size_t)(smem + base + ATile::dst_byte(w, j)));
#pragma unroll
            for (int j = 0; j < BTile::kPerWave; ++j)
                load16_to_lds_saddr(gb, b_src[j], (uint32_t)(size_t)(smem + base + A_BYTES + BTile::dst_byte(w, j)));
        } else {
#pragma unroll
            for (int j = 0; j < ATile::kPerWave; ++j)
                staged16(ga + a_src[j], base + ATile::dst_byte(w, j));
#pragma unroll
            for (int j = 0; j < BTile::kPerWave; ++j)
                staged16(gb + b_src[j], base + A_BYTES + BTile::dst_byte(w, j));
        }
        if (++ld_kb == kblocks) {
            ld_kb = 0;
            ++ld_i;
            if (p.A_off && ld_i < (int)p.batch) {
                ld_a = uniform_ptr(p.A + offs_a.get(ld_i, lane) + a_origin);
                ld_b = uniform_ptr(p.B + offs_b.get(ld_i, lane) + b_origin);
            }
        } else {
            ld_a += a_kstep;
            ld_b += b_kstep;
        }
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[a][b][r] = 0.0f;

    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int stage, int ks, int buf) {
        LDS_AS char *at = smem + (uint32_t)stage * STAGE;
        LDS_AS char *bt = at + A_BYTES;
#pragma unroll
        for (int t = 0; t < TM; ++t)
            fa[buf][t] = ATile::read_frag(at, wm * WM, t, ks, lane);
#pragma unroll
        for (int t = 0; t < TN; ++t)
            fb[buf][t] = BTile::read_frag(bt, wn * WN, t, ks, lane);
    };
    // Operands are passed swapped (B fragment first) so that the 32x32 result tile is
    // C^T: lane l then owns row m = l%32 and, per group of 4 registers, 4 consecutive
    // columns n - which makes the epilogue's stores 8 or 16 bytes per lane.
    auto mma = [&](int buf) {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b)
                acc[a][b] = mfma_32x32x16<KIND>(fb[buf][a], fa[buf][b], acc[a][b]);
    };

    if (n_iter > 0) {
        issue_loads(0);
        wait_vmcnt0();
        __syncthreads();
        if (n_iter > 1)
            issue_loads(1);
        read_frags(0, 0, 0);

        // Steady state; the last block is peeled so that the loop body has no branch
        // around the barrier (the same peeling the paper applies to its pipelined
        // packing loop).  Order inside one block: slices 0-2 multiply while the next
        // slice's fragments are read; before slice 3 is multiplied the barrier proves
        // block it+1 complete and block `it` fully read, then the request for block
        // it+2 and the first fragment reads of block it+1 are issued, and slice 3's
        // MFMAs cover their latency.
        for (int it = 0; it < n_iter - 1; ++it) {
            const int cur = it & 1;
            read_frags(cur, 1, 1);
            mma(0);
            read_frags(cur, 2, 0);
            mma(1);
            read_frags(cur, 3, 1);
            mma(0);
            wait_vmcnt0();
            wait_lgkmcnt0();
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            if (it + 2 < n_iter)
                issue_loads(cur);
            read_frags(cur ^ 1, 0, 0);
            mma(1);
        }
        {
            const int cur = (n_iter - 1) & 1;
            read_frags(cur, 1, 1);
            mma(0);
            read_frags(cur, 2, 0);
            mma(1);
            read_frags(cur, 3, 1);
            mma(0);
            mma(1);
        }
    }

    // ---- epilogue: beta*C, bias, ReLU, narrowing, store (or raw partial for a split)
    // Every accumulator index below is a compile-time constant (static_for), so the
    // tile never leaves the register file.
    store_wave_tile<TM, TN>(p, acc, m0 + wm * WM + (lane & 31), n0 + wn * WN + 4 * (lane >> 5), (int)blockIdx.y);
}

// ---------------------------------------------------------------------------

template <int BM, int BN>
static hipError_t launch_tile(const Problem &p)
{
    Bf16Args a;
    fill_common_args(a, p);
    a.tiles_m = (int)((p.M + BM - 1) / BM);
    a.tiles_n = (int)((p.N + BN - 1) / BN);
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)p.split, (unsigned)p.nmat);
    const size_t lds = 2 * (size_t)(BM + BN) * BK * 2;
    const bool ak = p.transA == 0;
    const int lay = p.b_packed ? LAY_PACKED : (p.transB == 1 ? LAY_K : LAY_MN);
    void (*kern)(Bf16Args) = nullptr;
#define BRG_PICK(KIND)                                                                        \
    if (ak && lay == LAY_K) kern = bf16_mfma_kernel<BM, BN, true, LAY_K, KIND>;                \
    else if (ak && lay == LAY_MN) kern = bf16_mfma_kernel<BM, BN, true, LAY_MN, KIND>;         \
    else if (ak) kern = bf16_mfma_kernel<BM, BN, true, LAY_PACKED, KIND>;                      \
    else if (lay == LAY_K) kern = bf16_mfma_kernel<BM, BN, false, LAY_K, KIND>;                \
    else if (lay == LAY_MN) kern = bf16_mfma_kernel<BM, BN, false, LAY_MN, KIND>;              \
    else kern = bf16_mfma_kernel<BM, BN, false, LAY_PACKED, KIND>;
    if (p.in_s8) {
        if (ak) kern = lay == LAY_K ? bf16_mfma_kernel<BM, BN, true, LAY_K, KIND_S8> : bf16_mfma_kernel<BM, BN, true, LAY_MN, KIND_S8>;
        else kern = lay == LAY_K ? bf16_mfma_kernel<BM, BN, false, LAY_K, KIND_S8> : bf16_mfma_kernel<BM, BN, false, LAY_MN, KIND_S8>;
    } else if (p.in_f16) { BRG_PICK(KIND_F16) } else { BRG_PICK(KIND_BF16) }
#undef BRG_PICK
    static thread_local const void *configured[16] = {nullptr};
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
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, p.stream, a);
    return hipGetLastError();
}

hipError_t launch_bf16_128x128(const Problem &p) { return launch_tile<128, 128>(p); }

// Alignment and shape rules of the kernels in this file.
bool bf16_mfma_eligible(const Problem &p)
{
    if (in_8bit(p)) {
        // one-byte elements: whole 128-deep k-blocks, 16-byte aligned rows, and whole 16-byte
        // chunks along m / n where that is the contiguous direction
        if (p.transA == 1 && (p.M & 15))
            return false;
        if (p.transB == 0 && (p.N & 15))
            return false;
        return !p.b_packed && p.batch == 1 && !p.A_off && !p.B_off && p.nmat == 1 &&
               p.K % 128 == 0 && !((uintptr_t)p.A & 15) && !((uintptr_t)p.B & 15) && !(p.lda & 15) &&
               !(p.ldb & 15) && p.lda < (1 << 23) && p.ldb < (1 << 23) && p.K / 128 < ((int64_t)1 << 31) &&
               p.M * p.N < ((int64_t)1 << 40);
    }
    if (!in_16bit(p))
        return false;
    if (p.K % BK != 0)
        return false;
    if (((uintptr_t)p.A & 15) || ((uintptr_t)p.B & 15) || (p.lda & 7) || (p.ldb & 7))
        return false;
    if ((p.ms_a & 7) || (p.ms_b & 7))          // every matrix of a batched call starts 16-byte aligned
        return false;
    if (p.transA == 1 && (p.M & 7))
        return false;
    if (!p.b_packed && p.transB == 0 && (p.N & 7))
        return false;
    if (p.lda >= (1 << 22) || p.ldb >= (1 << 22))
        return false;
    if (p.batch * (p.K / BK) >= ((int64_t)1 << 31) || p.M * p.N >= ((int64_t)1 << 40))
        return false;
    return true;
}

}  // namespace brg
