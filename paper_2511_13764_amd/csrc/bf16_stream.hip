// bf16 GEMM kernels for few rows of A (skinny M: the M = 16 / 128 shapes of an MLP
// layer), where the time goes into streaming the B matrix from HBM once, not into the
// matrix pipe - the regime the paper describes as bound by memory bandwidth
// (Section 6, discussion of the flat-layout results) - and for grids of at most 256
// tiles of 128 x 128 (one workgroup per CU anyway: the 1024^3 and 2048^3 squares, the
// batch-reduce tiles).
//
// bf16_stream_kernel: a workgroup of 4 or 8 wavefronts owns a BM x 128 block of C
// (BM = 32 or 64; 128 only for FP8) and walks its share of K in 64-deep blocks.  What
// matters here is how many bytes are in flight per CU, so the LDS is a ring of three
// stages, each holding one k-block of A and B: the loads for block t + 2 are requested
// while block t is multiplied, and the small footprint (60 to 96 KiB) lets a second
// workgroup share the CU.  (Sweeps of 2 to 8 stages on the MLP shapes: three is best
// or within 3 % of the best everywhere; deeper rings lose the second workgroup and
// gain nothing.)  Loads are global->LDS DMA (no register staging), counted per wave
// with vmcnt: before block t is read a wave waits until only the loads of block t + 1
// are outstanding, then one workgroup barrier publishes the block and frees the slot
// read in the previous iteration.
//
// bf16_stream128_kernel: the 128-row tile, with loading and multiplying given to
// different waves (described at the kernel).
#include "bf16_tiles.hpp"

namespace brg {

namespace {

constexpr int ST_BN = 128;
constexpr int ST_STAGES = 3;

// Waves per workgroup: 8 (two per SIMD) for the 128- and 64-row tiles - twice as many
// waves issuing the global->LDS loads raises what one CU can pull (measured 77-96
// against 57 B/ns) and these shapes are bound by exactly that; 4 for the 32-row tile,
// whose A block is only 4 wave-loads.
template <int BM>
struct StreamWaves { static constexpr int value = BM >= 64 ? 8 : 4; };

// STAGES: depth of the LDS ring (three, see above; a six-deep ring for batch-reduce
// calls over scattered tiles measured the same as three: there the time is a chain of
// fixed latencies - launch, offsets, first tiles, partial tiles, second launch).
template <int BM, bool A_KMAJ, int B_LAY, int KIND, int STAGES = ST_STAGES>
__global__ void __launch_bounds__(StreamWaves<BM>::value * 64)
bf16_stream_kernel(Bf16Args p)
{
    constexpr int NW = StreamWaves<BM>::value;
    static_assert(A_KMAJ || BM == 128, "an m-contiguous A needs the 128-row tile");
    typedef typename TileOf<BM, NW, A_KMAJ ? LAY_K : LAY_MN, KIND>::type ATile;
    typedef typename TileOf<ST_BN, NW, B_LAY, KIND>::type BTile;
    constexpr int WGM = BM == 128 ? 2 : 1, WGN = NW / WGM;    // wave grid
    constexpr int WM = BM / WGM, WN = ST_BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;                 // 16x16 MFMA tiles per wave
    constexpr uint32_t A_BYTES = BM * BK * 2, B_BYTES = ST_BN * BK * 2;
    constexpr uint32_t STAGE = A_BYTES + B_BYTES;
    constexpr int L = ATile::kPerWave + BTile::kPerWave;        // loads per wave per block
    constexpr int stages = STAGES;
    static_assert((STAGES - 2) * L <= 63, "outstanding loads must fit vmcnt");

    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    LDS_AS char *smem = (LDS_AS char *)smem_generic;
    select_matrix(p);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / WGN, wn = w % WGN;

    int tile, slice;
    slice_major_coords(p.tiles_m * p.tiles_n, tile, slice);
    const int tm = tile % p.tiles_m, tn = tile / p.tiles_m;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * ST_BN;

    // Reduction range of this workgroup: flattened (batch, k-block) iterations.
    const int kblocks = (int)(p.K / BK);
    const int total = (int)p.batch * kblocks;
    const int per = (total + p.split - 1) / p.split;
    const int it_begin = slice * per;
    const int it_end = (it_begin + per < total) ? it_begin + per : total;
    const int n_iter = it_end > it_begin ? it_end - it_begin : 0;

    // Rows / columns past the edge of the matrix are redirected to a valid one (their
    // products land in accumulator rows / columns that are never stored), so every
    // wave issues exactly L loads per block and the vmcnt arithmetic below holds.
    uint32_t a_src[ATile::kPerWave], b_src[BTile::kPerWave];
#pragma unroll
    for (int j = 0; j < ATile::kPerWave; ++j)
        a_src[j] = ATile::src_rel_bytes(w, j, lane, m0, p.M, p.lda);
#pragma unroll
    for (int j = 0; j < BTile::kPerWave; ++j)
        b_src[j] = BTile::src_rel_bytes(w, j, lane, n0, p.N, p.ldb);
    const int64_t b_kstep = BTile::kstep(p.ldb);
    const int64_t a_kstep = ATile::kstep(p.lda);
    const int64_t a_origin = ATile::origin(m0, p.lda), b_origin = BTile::origin(n0, p.ldb);
    // Load cursor: (batch index, k-block) of the next block to request and its pointers.
    int ld_i = n_iter > 0 ? it_begin / kblocks : 0;
    int ld_kb = n_iter > 0 ? it_begin - ld_i * kblocks : 0;
    TileOffsets offs_a, offs_b;                 // this wave's window of the tile offsets
    // Tile offsets live in device memory: if one of this workgroup's tiles does not
    // start at a multiple of 8 elements the workgroup stages its blocks through
    // registers with 2-byte loads instead (same LDS image; those loads complete before
    // the stores, so the counted waits below simply find nothing outstanding).  Every
    // wave looks at all of the workgroup's tiles (the first 64 are the window it keeps),
    // so all waves reach the same verdict without a barrier.
    bool direct = true;
    if (p.A_off) {
        offs_a.init(p.A_off, p.batch, ld_i, lane);
        offs_b.init(p.B_off, p.batch, ld_i, lane);
        const int last_i = n_iter > 0 ? (it_end - 1) / kblocks : ld_i;
        int bad = (ld_i + lane <= last_i) && (((offs_a.lo | offs_b.lo) & 7u) != 0);
        for (int i = ld_i + 64 + lane; i <= last_i; i += 64)
            bad |= (((p.A_off[i] | p.B_off[i]) & 7) != 0);
        direct = __builtin_amdgcn_ballot_w64(bad != 0) == 0;
    }
    const uint16_t *ld_a = uniform_ptr(p.A + (p.A_off ? offs_a.get(ld_i, lane) : 0) + a_origin + ld_kb * a_kstep);
    const uint16_t *ld_b = uniform_ptr(p.B + (p.B_off ? offs_b.get(ld_i, lane) : 0) + b_origin + ld_kb * b_kstep);
    int ld_slot = 0;
    auto staged16 = [&](const char *gc, uint32_t lds_byte) {
        const uint16_t *g = (const uint16_t *)gc;
        s16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = (short)g[e];
        *(LDS_AS s16x8 *)(smem + lds_byte + lane * 16) = v;
    };

    auto issue_loads = [&]() {
        const uint32_t base = (uint32_t)ld_slot * STAGE;
        if (direct) {
#pragma unroll
            for (int j = 0; j < BTile::kPerWave; ++j)
                load16_to_lds_saddr((const char *)ld_b, b_src[j],
                                    (uint32_t)(size_t)(smem + base + A_BYTES + BTile::dst_byte(w, j)));
#pragma unroll
            for (int j = 0; j < ATile::kPerWave; ++j)
                load16_to_lds_saddr((const char *)ld_a, a_src[j],
                                    (uint32_t)(size_t)(smem + base + ATile::dst_byte(w, j)));
        } else {
#pragma unroll
            for (int j = 0; j < BTile::kPerWave; ++j)
                staged16((const char *)ld_b + b_src[j], base + A_BYTES + BTile::dst_byte(w, j));
#pragma unroll
            for (int j = 0; j < ATile::kPerWave; ++j)
                staged16((const char *)ld_a + a_src[j], base + ATile::dst_byte(w, j));
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
        ld_slot = ld_slot + 1 == stages ? 0 : ld_slot + 1;
    };
    f32x4 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
            acc[a][b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int ahead = stages - 1;
    for (int s = 0; s < ahead && s < n_iter; ++s)
        issue_loads();

    // The MFMAs of the second 32-deep half of a block are issued at the top of the next
    // iteration, so the matrix pipe works through the wait for the next block, the barrier
    // and the load requests.  (Not for FP8: its 128-deep instruction needs both halves.)
    bf16x8 fa[2][TM], fb[2][TN];
    auto mfma_half = [&](auto hc) {
        constexpr int h = decltype(hc)::value;
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b)
                acc[a][b] = mfma_16x16x32<kind_is_f8(KIND) ? KIND_BF16 : KIND>(fb[h][a], fa[h][b], acc[a][b]);
    };
    constexpr std::integral_constant<int, 0> H0{};
    constexpr std::integral_constant<int, 1> H1{};
    int rd_slot = 0;
    for (int t = 0; t < n_iter; ++t) {
        if constexpr (!kind_is_f8(KIND)) {
            if (t > 0)
                mfma_half(H1);                      // second half of block t - 1
            __builtin_amdgcn_sched_barrier(0);
        }
        // Block t has landed once only the stages - 2 younger blocks are outstanding.
        if (t + stages - 2 < n_iter)
            wait_vmcnt_le<(STAGES - 2) * L>();
        else
            wait_vmcnt0();                          // tail: fewer blocks than slots remain
        if (!direct)
            wait_lgkmcnt0();                        // register-staged blocks: their LDS stores
        block_sync();
        if (t + ahead < n_iter)
            issue_loads();                          // into the slot read in iteration t - 1
        LDS_AS char *at = smem + (uint32_t)rd_slot * STAGE;
        LDS_AS char *bt = at + A_BYTES;
#pragma unroll
        for (int st = 0; st < 2; ++st) {
#pragma unroll
            for (int i = 0; i < TM; ++i)            // FP8: st = which half of a lane's 32-byte operand
                fa[st][i] = ATile::read_frag16(at, wm * WM, i, st, lane);
#pragma unroll
            for (int i = 0; i < TN; ++i)
                fb[st][i] = BTile::read_frag16(bt, wn * WN, i, st, lane);
        }
        if constexpr (kind_is_f8(KIND)) {
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    acc[a][b] = mfma_16x16x128_f8<KIND>(fb[0][a], fb[1][a], fa[0][b], fa[1][b], acc[a][b]);
        } else {
            mfma_half(H0);
        }
        // The fragments are in registers before the next barrier lets another wave's
        // loads overwrite this slot.
        wait_lgkmcnt0();
        rd_slot = rd_slot + 1 == stages ? 0 : rd_slot + 1;
    }
    if constexpr (!kind_is_f8(KIND)) {
        if (n_iter > 0)
            mfma_half(H1);
    }

    store_wave_tile16<TM, TN>(p, acc, m0 + wm * WM + (lane & 15), n0 + wn * WN + 4 * (lane >> 4), slice);
}

// ---------------------------------------------------------------------------
// 128 x 128 tile with the work divided by kind: four waves multiply, four waves load.
//
// What bounds a 128 x 128 x 64 block on one CU (cycles per block, measured with
// work-skipping copies of the kernel above and with s_memtime around its steps):
// the matrix pipe needs 512 per SIMD; eight waves reading the fragments of 64 x 32
// accumulator tiles need 600-1100 (96 KiB of LDS reads, a SIMD takes its share at
// about 32 B/clk); the 32 global->LDS wave-loads need about 780 (a CU pulls at
// most ~42 B/clk from L2 with every CU pulling), and a wave is held at each of its
// loads until the address unit has taken it.  In the kernel above all of that is
// serial: every wave requests loads, reads fragments, then multiplies - 0.63 us per
// block where the loads alone need 0.34.
//
// Here waves 0-3 (one per SIMD) own 64 x 64 accumulator tiles (64 KiB of fragment
// reads per block) and never touch global memory inside the loop; waves 4-7 (the
// second wave of every SIMD) only request loads, eight per block each, and wait
// for them.  One workgroup barrier per block, B(t), publishes block t and frees
// the slot of block t - 1, into which the loaders then request block t + STAGES - 1.
// A multiplying wave reads the fragments of the first 32-deep half of block t
// while the matrix pipe works on the second half of block t - 1, and those of the
// second half while it works on the first, so the pipe only idles for the barrier.
// ---------------------------------------------------------------------------
#ifndef BRG_ST128_STAGES
#define BRG_ST128_STAGES 4
#endif
constexpr int S128_STAGES = BRG_ST128_STAGES;

constexpr int S128_EPI_LD = ST_BN + 4;           // floats per staged row (528 B: conflict-free 16-byte writes)

// All 512 threads: the staged 128 x 128 fp32 tile, two rows per wave and instruction, to
// C (beta, bias, ReLU, narrowing) or to this split's partial sums.
__device__ __forceinline__ void stream128_store_tile(const Bf16Args &p, LDS_AS char *smem, int tid, int64_t m0, int64_t n0,
                                                     int slice)
{
    LDS_AS float *stage = (LDS_AS float *)smem;
    const bool to_partial = p.split > 1;
    float *part = to_partial ? p.partial + (int64_t)slice * p.M * p.N : nullptr;
    const bool vec = to_partial ? ((p.N & 3) == 0) : ((p.epi.ldc & 3) == 0 && (((uintptr_t)p.epi.C) & 15) == 0);
#pragma unroll 2
    for (int i = 0; i < 8; ++i) {
        const int idx = i * 512 + tid;
        const int row = idx >> 5, c4 = idx & 31;
        const f32x4 v = *(LDS_AS f32x4 *)(stage + row * S128_EPI_LD + c4 * 4);
        const int64_t m = m0 + row, n = n0 + c4 * 4;
        if (m < p.M && n < p.N) {
            if (to_partial)
                store4_partial(part + m * p.N + n, p.N - n, vec, v[0], v[1], v[2], v[3]);
            else
                store4_epilogue(p.epi, m, n, p.N - n, vec, v[0], v[1], v[2], v[3]);
        }
    }
}

template <bool A_KMAJ, int B_LAY, int KIND>
__global__ void __launch_bounds__(512)
bf16_stream128_kernel(Bf16Args p)
{
    constexpr int BM = 128, NL = 4;              // NL: loader waves
    static_assert(!kind_is_f8(KIND), "the 128-deep FP8 instruction takes a whole k-block");
    typedef typename TileOf<BM, NL, A_KMAJ ? LAY_K : LAY_MN, KIND>::type ATile;
    typedef typename TileOf<ST_BN, NL, B_LAY, KIND>::type BTile;
    constexpr int WM = 64, WN = 64, TM = WM / 16, TN = WN / 16;
    constexpr uint32_t A_BYTES = BM * BK * 2, B_BYTES = ST_BN * BK * 2;
    constexpr uint32_t STAGE = A_BYTES + B_BYTES;
    constexpr int LA = ATile::kPerWave, LB = BTile::kPerWave, L = LA + LB;
    constexpr int stages = S128_STAGES, ahead = stages - 1;
    static_assert(L == 8 && (stages - 2) * L <= 63, "outstanding loads must fit vmcnt");

    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    LDS_AS char *smem = (LDS_AS char *)smem_generic;
    select_matrix(p);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    int tile, slice, tm, tn;
    slice_major_coords(p.tiles_m * p.tiles_n, tile, slice);
    group_walk(tile, p.tiles_m, p.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * ST_BN;

    const int kblocks = (int)(p.K / BK);
    const int total = (int)p.batch * kblocks;
    const int per = (total + p.split - 1) / p.split;
    const int it_begin = slice * per;
    const int it_end = (it_begin + per < total) ? it_begin + per : total;
    const int n_iter = it_end > it_begin ? it_end - it_begin : 0;

    // A tile offset that is not a multiple of 8 elements sends the loaders to
    // register-staged 2-byte loads (same LDS image; they complete before their LDS
    // stores, so the counted waits find nothing outstanding).
    bool direct = true;
    if (p.A_off) {
        int ok = 1;
        for (int i = tid; i < (int)p.batch; i += 512)
            ok &= (((p.A_off[i] | p.B_off[i]) & 7) == 0);
        direct = __syncthreads_and(ok) != 0;
    }

    if (w >= 4) {
        // ---------------- loader waves ----------------
        const int wl = w - 4;
        // Rows / columns past the edge are redirected to a valid one (their products
        // land in accumulator rows / columns that are never stored), so every wave
        // issues exactly L loads per block and the vmcnt arithmetic holds.
        uint32_t a_src[LA], b_src[LB];
#pragma unroll
        for (int j = 0; j < LA; ++j)
            a_src[j] = ATile::src_rel_bytes(wl, j, lane, m0, p.M, p.lda);
#pragma unroll
        for (int j = 0; j < LB; ++j)
            b_src[j] = BTile::src_rel_bytes(wl, j, lane, n0, p.N, p.ldb);
        const int64_t b_kstep = BTile::kstep(p.ldb);
        const int64_t a_kstep = ATile::kstep(p.lda);
        const int64_t a_origin = ATile::origin(m0, p.lda), b_origin = BTile::origin(n0, p.ldb);
        int ld_i = n_iter > 0 ? it_begin / kblocks : 0;
        int ld_kb = n_iter > 0 ? it_begin - ld_i * kblocks : 0;
        TileOffsets offs_a, offs_b;             // this wave's window of the tile offsets
        if (p.A_off) {
            offs_a.init(p.A_off, p.batch, ld_i, lane);
            offs_b.init(p.B_off, p.batch, ld_i, lane);
        }
        const uint16_t *ld_a = uniform_ptr(p.A + (p.A_off ? offs_a.get(ld_i, lane) : 0) + a_origin + ld_kb * a_kstep);
        const uint16_t *ld_b = uniform_ptr(p.B + (p.B_off ? offs_b.get(ld_i, lane) : 0) + b_origin + ld_kb * b_kstep);
        int ld_slot = 0;
        auto issue_one = [&](const char *base, uint32_t src, uint32_t dst) {
            if (direct) {
                load16_to_lds_saddr(base, src, (uint32_t)(size_t)(smem + dst));
            } else {
                const uint16_t *h = (const uint16_t *)(base + src);
                s16x8 v;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (short)h[e];
                *(LDS_AS s16x8 *)(smem + dst + lane * 16) = v;
            }
        };
        auto issue_block = [&]() {
            const uint32_t base = (uint32_t)ld_slot * STAGE;
#pragma unroll
            for (int j = 0; j < LB; ++j)
                issue_one((const char *)ld_b, b_src[j], base + A_BYTES + BTile::dst_byte(wl, j));
#pragma unroll
            for (int j = 0; j < LA; ++j)
                issue_one((const char *)ld_a, a_src[j], base + ATile::dst_byte(wl, j));
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
            ld_slot = ld_slot + 1 == stages ? 0 : ld_slot + 1;
        };
        for (int s = 0; s < ahead && s < n_iter; ++s)
            issue_block();
        for (int t = 0; t < n_iter; ++t) {
            // Block t has landed once only the stages - 2 younger blocks are outstanding.
            if (t + ahead - 1 < n_iter)
                wait_vmcnt_le<(stages - 2) * L>();
            else
                wait_vmcnt0();                      // tail: fewer blocks than slots remain
            wait_lgkmcnt0();                        // register-staged blocks: their LDS stores
            block_sync();                           // B(t)
            if (t + ahead < n_iter)
                issue_block();                      // into the slot of block t - 1
        }
        block_sync();                               // E1
        block_sync();                               // E2: the staged tile is complete
        stream128_store_tile(p, smem, tid, m0, n0, slice);
        return;
    }

    // ---------------- multiplying waves ----------------
    const int wm = w >> 1, wn = w & 1;
    f32x4 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
            acc[a][b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_half = [&](LDS_AS char *at, LDS_AS char *bt, auto hc) {
        constexpr int h = decltype(hc)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[h][i] = ATile::read_frag16(at, wm * WM, i, h, lane);
#pragma unroll
        for (int i = 0; i < TN; ++i)
            fb[h][i] = BTile::read_frag16(bt, wn * WN, i, h, lane);
    };
    auto mfma_half = [&](auto hc) {
        constexpr int h = decltype(hc)::value;
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b)
                acc[a][b] = mfma_16x16x32<KIND>(fb[h][a], fa[h][b], acc[a][b]);
    };
    constexpr std::integral_constant<int, 0> H0{};
    constexpr std::integral_constant<int, 1> H1{};
    int rd_slot = 0;
    for (int t = 0; t < n_iter; ++t) {
        block_sync();                               // B(t): block t is in LDS
        LDS_AS char *at = smem + (uint32_t)rd_slot * STAGE;
        LDS_AS char *bt = at + A_BYTES;
        read_half(at, bt, H0);
        if (t > 0)
            mfma_half(H1);                          // second half of block t - 1
        __builtin_amdgcn_sched_barrier(0);
        read_half(at, bt, H1);
        mfma_half(H0);
        __builtin_amdgcn_sched_barrier(0);
        // Every read of block t is complete before the barrier that lets the loaders
        // overwrite its slot.
        wait_lgkmcnt0();
        rd_slot = rd_slot + 1 == stages ? 0 : rd_slot + 1;
    }
    if (n_iter > 0)
        mfma_half(H1);
    // Epilogue through LDS: written from the MFMA layout (lane l: row l % 16, columns
    // 4 * (l / 16) .. + 3 of each 16 x 16 tile), read back row-wise by all eight waves,
    // so that every store instruction covers whole rows of the tile instead of sixteen
    // 32-byte pieces (measured: 4 us of an 8 MiB C went into such stores).
    block_sync();                                   // E1: nobody reads fragments any more
    LDS_AS float *stage = (LDS_AS float *)smem;
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
            *(LDS_AS f32x4 *)(stage + (wm * WM + 16 * b + (lane & 15)) * S128_EPI_LD + wn * WN + 16 * a + 4 * (lane >> 4)) =
                acc[a][b];
    wait_lgkmcnt0();
    block_sync();                                   // E2
    stream128_store_tile(p, smem, tid, m0, n0, slice);
}

template <int BM>
hipError_t launch_stream(const Problem &p)
{
    Bf16Args a;
    fill_common_args(a, p);
    a.tiles_m = (int)((p.M + BM - 1) / BM);
    a.tiles_n = (int)((p.N + ST_BN - 1) / ST_BN);
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)p.split, (unsigned)p.nmat);
    void (*kern)(Bf16Args) = nullptr;
    size_t lds = (size_t)ST_STAGES * (BM + ST_BN) * BK * 2;
    // One-byte operands come unpacked in all four layouts; 16-bit ones also with a packed B.
#define BRG_ST_B(AK, KIND)                                                                    \
    kern = p.transB == 1 ? bf16_stream_kernel<BM, AK, LAY_K, KIND> : bf16_stream_kernel<BM, AK, LAY_MN, KIND>;
#define BRG_ST_B3(AK, KIND)                                                                   \
    kern = p.b_packed ? bf16_stream_kernel<BM, AK, LAY_PACKED, KIND>                           \
           : p.transB == 1 ? bf16_stream_kernel<BM, AK, LAY_K, KIND> : bf16_stream_kernel<BM, AK, LAY_MN, KIND>;
#define BRG_S128_B(AK, KIND)                                                                  \
    kern = p.transB == 1 ? bf16_stream128_kernel<AK, LAY_K, KIND> : bf16_stream128_kernel<AK, LAY_MN, KIND>;
#define BRG_S128_B3(AK, KIND)                                                                 \
    kern = p.b_packed ? bf16_stream128_kernel<AK, LAY_PACKED, KIND>                            \
           : p.transB == 1 ? bf16_stream128_kernel<AK, LAY_K, KIND> : bf16_stream128_kernel<AK, LAY_MN, KIND>;
    if constexpr (BM == 128) {
        // Everything but FP8 takes the loader / multiplier form of the 128-row tile.
        if (p.in_f8) {
            if (p.transA == 0) {
                if (p.f8_e5m2) { BRG_ST_B(true, KIND_BF8) } else { BRG_ST_B(true, KIND_F8) }
            } else {
                if (p.f8_e5m2) { BRG_ST_B(false, KIND_BF8) } else { BRG_ST_B(false, KIND_F8) }
            }
        } else {
            lds = (size_t)S128_STAGES * (BM + ST_BN) * BK * 2;
            if (p.transA == 0) {
                if (p.in_s8) { BRG_S128_B(true, KIND_S8) }
                else if (p.in_f16) { BRG_S128_B3(true, KIND_F16) } else { BRG_S128_B3(true, KIND_BF16) }
            } else {
                if (p.in_s8) { BRG_S128_B(false, KIND_S8) }
                else if (p.in_f16) { BRG_S128_B3(false, KIND_F16) } else { BRG_S128_B3(false, KIND_BF16) }
            }
        }
    } else {
        if (p.transA != 0)
            return hipErrorInvalidValue;            // the 32- and 64-row tiles need a k-contiguous A
        if (p.in_s8) {
            BRG_ST_B(true, KIND_S8)
        } else if (p.in_f8) {
            if (p.f8_e5m2) { BRG_ST_B(true, KIND_BF8) } else { BRG_ST_B(true, KIND_F8) }
        } else if (p.in_f16) {
            BRG_ST_B3(true, KIND_F16)
        } else {
            BRG_ST_B3(true, KIND_BF16)
        }
    }
#undef BRG_ST_B
#undef BRG_ST_B3
#undef BRG_S128_B
#undef BRG_S128_B3
    static thread_local const void *configured[40] = {nullptr};
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
    hipLaunchKernelGGL(kern, grid, dim3(StreamWaves<BM>::value * 64), lds, p.stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bf16_stream(const Problem &p, int bm)
{
    switch (bm) {
    case 32: return launch_stream<32>(p);
    case 64: return launch_stream<64>(p);
    case 128: return launch_stream<128>(p);
    default: return hipErrorInvalidValue;
    }
}

// The 32- and 64-row tiles need A stored M x K (k contiguous), the 128-row tile takes
// either order; B in any layout; batch-reduce with tile offsets included.
bool bf16_stream_eligible(const Problem &p, int bm)
{
    return bf16_mfma_eligible(p) && (p.transA == 0 || bm == 128);
}

}  // namespace brg
