// bf16 BRGEMM kernel for gfx950 with two wavefronts per SIMD working in
// alternating phases ("ping-pong"): 256 x 256 x 64 workgroup tile, 8 wavefronts,
// each keeping a 128 x 64 accumulator tile in registers for the whole batch and K
// loops (Section 2.1 advantage (1); Section 3.1: the register tile is sized so that
// accumulators, the operand fragments of one phase and the load addresses fit the
// 256 registers a lane has at this occupancy, with no spills).
//
// Why two waves per SIMD: a global->LDS load holds the issuing wave until the
// address unit has taken it (about 15 cycles per 1 KiB wave-load per CU, i.e. the
// 64 B/clk of the vector memory path), and the 64 loads a k-block needs occupy
// that unit for about half of the block's MFMA time.  With one wave per SIMD that
// time is lost to the matrix pipe; here one wave of each SIMD issues loads and LDS
// fragment reads ("memory phase") while the other issues nothing but its 64 MFMAs
// ("compute phase"), and a workgroup barrier swaps the roles.  Waves 4-7 run the
// same sequence one phase behind waves 0-3.  It is the software pipelining of
// operand re-layout against the matrix instruction that the paper applies to its
// flat-layout AMX kernels (Section 4.3), done across waves.
//
// LDS holds five 32 KiB slots used as a ring of half-blocks A(0) B(0) A(1) B(1) ...
// With five slots the A half of block t+2 has a free slot while block t is still
// being read, so every load is requested at least one and a half phases (~1500
// cycles) before the barrier that publishes it: waves 0-3 request B(t+1) in their
// memory phase of block t, waves 4-7 request A(t+2) in theirs.
#pragma once
#include "bf16_tiles.hpp"

namespace brg {

namespace {

constexpr int PP_BM = 256, PP_BN = 256, PP_NW = 8;
constexpr int PP_WM = 128, PP_WN = 64;          // wave tile
constexpr int PP_TM = PP_WM / 16, PP_TN = PP_WN / 16;     // 16x16 MFMA tiles per wave tile: 8 x 4
constexpr uint32_t PP_A_BYTES = PP_BM * BK * 2, PP_B_BYTES = PP_BN * BK * 2;
constexpr uint32_t PP_SLOT = 32768;              // one half-block (A or B part of a k-block)
constexpr int PP_SLOTS = 5;
static_assert(PP_A_BYTES == PP_SLOT && PP_B_BYTES == PP_SLOT, "half-blocks are one slot each");
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int PP_EPI_LD = PP_WN + 4;            // floats per staged epilogue row (272 B: conflict-free)

__device__ __forceinline__ void phase_sync()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

}  // namespace

// DIRECT: global->LDS DMA loads (false: register-staged 2-byte loads, for tile
// offsets that are not 16-byte aligned).  EDGE: the tile overhangs the matrix in the
// direction this wave loads, so lanes outside it are switched off.  Both are uniform
// over the workgroup / wave and chosen once, so the loop body carries no branches for them.
// HAS_OFF: a batch-reduce call with tile offsets.  A template argument so that the plain GEMM
// body carries none of the offset state (the kernel sits at 251-255 of 256 registers).
template <bool A_KMAJ, int B_LAY, bool DIRECT, bool EDGE, int KIND, bool HAS_OFF>
__device__ __forceinline__ void pp_body(const Bf16Args &p)
{
    // Load duty: waves 0-3 fetch the B halves, waves 4-7 the A halves (8 wave-loads
    // per half-block each), so the tile classes are instantiated for 4 loader waves.
    typedef typename TileOf<PP_BM, 4, A_KMAJ ? LAY_K : LAY_MN, KIND>::type ATile;
    typedef typename TileOf<PP_BN, 4, B_LAY, KIND>::type BTile;
    static_assert(ATile::kPerWave == 8 && BTile::kPerWave == 8, "8 wave-loads per loader wave");

    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    LDS_AS char *smem = (LDS_AS char *)smem_generic;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w & 1, wn = (w >> 1) & 3;
    const int group = w >> 2;                   // waves w and w+4 share a SIMD
    const int wl = w & 3;                       // index among the loaders of one operand

    int tm, tn;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * PP_BM, n0 = (int64_t)tn * PP_BN;

    const int kblocks = (int)(p.K / BK);
    const int total = (int)p.batch * kblocks;
    const int per = (total + p.split - 1) / p.split;
    const int it_begin = (int)blockIdx.y * per;
    const int it_end = (it_begin + per < total) ? it_begin + per : total;
    const int n_iter = it_end - it_begin;

    // This wave's operand (A for waves 4-7, B for waves 0-3).  A wave-load g of a
    // half-block is addressed as scalar base + a scalar offset of g + a 32-bit lane
    // offset that only depends on the parity of g (two registers for the whole kernel).
    const uint16_t *op_base = group ? p.A : p.B;
    const int64_t *op_off = group ? p.A_off : p.B_off;
    const int64_t op_ld = group ? p.lda : p.ldb;
    const int64_t op_first = group ? m0 : n0;             // first row / column of the tile
    const int64_t op_limit = group ? p.M : p.N;
    const int64_t op_origin = group ? ATile::origin(m0, p.lda) : BTile::origin(n0, p.ldb);
    const int64_t op_kstep = group ? ATile::kstep(p.lda) : BTile::kstep(p.ldb);
    // Wave-load g of a half-block (32 of them) is taken by loader wave wl as its j-th:
    //   g = (j & 3) | ((wl & 1) << 2) | ((2 * (wl >> 1) + (j >> 2)) << 3),
    // so bit 2 of g is the same for all 8 loads of a wave.  For an m/n-contiguous
    // operand that bit selects the second swizzle term (+-32 bytes per lane), which can
    // then be folded into the two lane offsets once instead of costing a register and
    // an add per load.
    const int g_fixed = (wl & 1) << 2;
    const int32_t fold = (group ? ATile::delta_applies(g_fixed) : BTile::delta_applies(g_fixed))
                             ? (group ? ATile::lane_delta_bytes(lane) : BTile::lane_delta_bytes(lane)) : 0;
    const uint32_t lane_off0 = (group ? ATile::lane_off_bytes(0, lane, op_ld) : BTile::lane_off_bytes(0, lane, op_ld)) + (uint32_t)fold;
    const uint32_t lane_off1 = (group ? ATile::lane_off_bytes(1, lane, op_ld) : BTile::lane_off_bytes(1, lane, op_ld)) + (uint32_t)fold;

    // Load cursor of this wave's operand: next block's (batch index, k-block), its
    // source pointer and its ring slot.  Half-block 2t is A(t), 2t+1 is B(t); slot = index % 5.
    int ld_i = n_iter > 0 ? it_begin / kblocks : 0;
    int ld_kb = n_iter > 0 ? it_begin - ld_i * kblocks : 0;
    // Tile offsets of a batch-reduce call: this wave's operand only, 64 at a time in two
    // registers (see TileOffsets: fetched one by one they would sit, as dependent vector
    // loads, in front of every tile's loads and drain the loads in flight).
    TileOffsets offs;
    if constexpr (HAS_OFF)
        offs.init(op_off, p.batch, ld_i, lane);
    int64_t first_off = 0;
    if constexpr (HAS_OFF)
        first_off = offs.get(ld_i, lane);
    const uint16_t *ld_ptr = uniform_ptr(op_base + first_off + op_origin + ld_kb * op_kstep);
    int ld_slot = group ? 0 : 1;

    // One of the 8 wave-loads of this wave's next half-block.
    auto issue_one = [&](int j) {
        const int gi = (j & 3) | g_fixed | ((2 * (wl >> 1) + (j >> 2)) << 3);
        const char *gj = (const char *)ld_ptr + (group ? ATile::instr_offset_bytes(gi, op_ld)
                                                       : BTile::instr_offset_bytes(gi, op_ld));
        const uint32_t off = (j & 1) ? lane_off1 : lane_off0;
        const uint32_t dst = (uint32_t)ld_slot * PP_SLOT + (uint32_t)gi * 1024u;
        const bool on = !EDGE || (group ? ATile::lane_valid(gi, lane, op_first, op_limit)
                                        : BTile::lane_valid(gi, lane, op_first, op_limit));
        if (on) {
            if constexpr (DIRECT) {
                load16_to_lds_saddr(gj, off, (uint32_t)(size_t)(smem + dst));
            } else {
                const uint16_t *h = (const uint16_t *)(gj + off);
                s16x8 v;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (short)h[e];
                *(LDS_AS s16x8 *)(smem + dst + lane * 16) = v;
            }
        }
    };
    auto advance_loads = [&]() {
        ld_slot = ld_slot + 2 >= PP_SLOTS ? ld_slot + 2 - PP_SLOTS : ld_slot + 2;
        if (++ld_kb == kblocks) {
            ld_kb = 0;
            ++ld_i;
            if constexpr (HAS_OFF) {
                if (ld_i < (int)p.batch)
                    ld_ptr = uniform_ptr(op_base + offs.get(ld_i, lane) + op_origin);
            }
        } else {
            ld_ptr += op_kstep;
        }
    };
    auto issue_half = [&]() {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            issue_one(j);
        advance_loads();
    };

    f32x4 acc[PP_TN][PP_TM];
#pragma unroll
    for (int a = 0; a < PP_TN; ++a)
#pragma unroll
        for (int b = 0; b < PP_TM; ++b)
            acc[a][b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // Memory phase: every fragment of one k-block (2 steps of 32 k; 8 + 4 fragments
    // each) into registers, and - when `request` - this wave's 8 loads of a later
    // half-block, one after every third fragment read so that the LDS reads complete
    // while the wave is held by the address unit.  The loads only write slots nobody
    // reads in this phase, so their order relative to the reads does not matter for
    // correctness.
    bf16x8 fa[2][PP_TM], fb[2][PP_TN];
    int rd_slot = 0;                            // slot of A(t); B(t) is the next one
    auto memory_phase = [&](bool request) {
        LDS_AS char *at = smem + (uint32_t)rd_slot * PP_SLOT;
        LDS_AS char *bt = smem + (uint32_t)(rd_slot + 1 == PP_SLOTS ? 0 : rd_slot + 1) * PP_SLOT;
        static_for<0, 8>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            static_for<0, 3>([&](auto ic) {
                constexpr int id = 3 * j + decltype(ic)::value;
                constexpr int st = id / (PP_TM + PP_TN), q = id % (PP_TM + PP_TN);
                // (FP8: the two reads are the halves of a lane's 32-byte operand, see read_frag16)
                if constexpr (q < PP_TM) {
                    fa[st][q] = ATile::read_frag16(at, wm * PP_WM, q, st, lane);
                } else {
                    fb[st][q - PP_TM] = BTile::read_frag16(bt, wn * PP_WN, q - PP_TM, st, lane);
                }
            });
            if (request)
                issue_one(j);
        });
        rd_slot = rd_slot + 2 >= PP_SLOTS ? rd_slot + 2 - PP_SLOTS : rd_slot + 2;
        if (request)
            advance_loads();
    };
    // Compute phase: 64 x v_mfma_f32_16x16x32_bf16 (the same 1024 matrix-pipe cycles as
    // 32 of the 32x32x16 form, but each accumulator register is read and written half as
    // often per flop: on random operands the register-only issue loop sustains ~15 %
    // more with this shape, and the chip is power-limited).  Operands are passed swapped
    // (B fragment first) so the 16x16 result is C^T: lane l owns row m = l%16 and the 4
    // consecutive columns 4*(l/16) .. +3.
    auto compute_block = [&]() {
        if constexpr (kind_is_f8(KIND)) {
            // one 128-deep instruction per accumulator: 32 MFMAs, the same pipe time
#pragma unroll
            for (int a = 0; a < PP_TN; ++a)
#pragma unroll
                for (int b = 0; b < PP_TM; ++b)
                    acc[a][b] = mfma_16x16x128_f8<KIND>(fb[0][a], fb[1][a], fa[0][b], fa[1][b], acc[a][b]);
            return;
        }
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int a = 0; a < PP_TN; ++a)
#pragma unroll
                for (int b = 0; b < PP_TM; ++b)
                    acc[a][b] = mfma_16x16x32<KIND>(fb[st][a], fa[st][b], acc[a][b]);
    };

    if (n_iter > 0) {
        // Prologue: A(0), A(1) by waves 4-7, B(0) by waves 0-3.
        issue_half();
        if (group == 1 && n_iter > 1)
            issue_half();
        wait_vmcnt0();
        wait_lgkmcnt0();
        phase_sync();
        if (group == 1)
            phase_sync();                       // waves 4-7 run one phase behind

        for (int t = 0; t < n_iter; ++t) {
            // ---- memory phase.  Waves 0-3 request B(t+1): its slot held A(t-1), last
            // read one phase ago.  Waves 4-7 request A(t+2): its slot held B(t-1).
            const bool request = group == 0 ? (t + 1 < n_iter) : (t + 2 < n_iter);
            memory_phase(request);
            wait_lgkmcnt0();
            if (group == 1) {
                // A(t+1), requested one block ago, must have landed before the barrier
                // that precedes its first read; the 8 loads just issued may still fly.
                // Counting is only valid when all 8 loads were really issued: on an edge
                // tile a wave-load whose lanes are all switched off is skipped entirely.
                if (request && !EDGE)
                    wait_vmcnt8();
                else
                    wait_vmcnt0();
            }
            phase_sync();
            // ---- compute phase
            compute_block();
            __builtin_amdgcn_sched_barrier(0);  // keep the wait behind the MFMAs
            if (group == 0)
                wait_vmcnt0();                  // B(t+1) has landed (requested a phase ago)
            phase_sync();
        }
        if (group == 0)
            phase_sync();
    }

    // ---- epilogue.  Each wave stages 32 rows x 64 columns of its tile at a time (two
    // rows of 16x16 accumulators) in its own 8.5 KiB of LDS (all stages are free now),
    // reads them back row-wise and stores 4 or 8 rows x whole cache lines per instruction.
    LDS_AS float *stage_f = (LDS_AS float *)(smem + (uint32_t)w * (32 * PP_EPI_LD * 4));
    const bool to_partial = p.split > 1;
    float *part = to_partial ? p.partial + (int64_t)blockIdx.y * p.M * p.N : nullptr;
    const bool vec = to_partial ? ((p.N & 3) == 0)
                                : ((p.epi.ldc & 3) == 0 && (((uintptr_t)p.epi.C) & 15) == 0);
    // Fast path for the common case (16-bit C, beta == 0, aligned, no overhang in N;
    // bias and ReLU - the fused kernel of Section 6 - included): bias and ReLU in
    // registers, narrowing with v_cvt_pk_bf16_f32, staging as 16-bit values (136-byte row
    // pitch: conflict-free 64-bit writes), read back 16 bytes per lane, 8 rows x 128
    // bytes per store instruction.
    const bool fast_bf16 = !to_partial && !p.epi.c_f32 && !p.epi.c_i32 && p.epi.beta == 0.0f &&
                           (p.epi.ldc & 7) == 0 && (((uintptr_t)p.epi.C) & 15) == 0 && n0 + PP_BN <= p.N;
    if (fast_bf16) {
        LDS_AS char *stage_h = smem + (uint32_t)w * (32 * 136);
        uint16_t *crow = (uint16_t *)p.epi.C + (m0 + wm * PP_WM) * p.epi.ldc + n0 + wn * PP_WN;
        // this lane's 4 columns of each of the 4 accumulator columns: 16 bias values
        f32x4 bias4[PP_TN];
        const bool has_bias = p.epi.bias != nullptr;
        const bool relu = p.epi.relu != 0;
        if (has_bias) {
            const float *bp = p.epi.bias + n0 + wn * PP_WN + 4 * (lane >> 4);
            const bool bvec = (((uintptr_t)p.epi.bias) & 15) == 0;
#pragma unroll
            for (int a = 0; a < PP_TN; ++a)
                bias4[a] = bvec ? *(const f32x4 *)(bp + 16 * a) : f32x4{bp[16 * a], bp[16 * a + 1], bp[16 * a + 2], bp[16 * a + 3]};
        }
        static_for<0, PP_TM / 2>([&](auto bc) {
            constexpr int b2 = decltype(bc)::value;
            asm volatile("" ::: "memory");
            static_for<0, 2 * PP_TN>([&](auto aq) {
                constexpr int bb = decltype(aq)::value / PP_TN, a = decltype(aq)::value % PP_TN;
                const int row = 16 * bb + (lane & 15);
                const int col = 16 * a + 4 * (lane >> 4);
                f32x4 v = acc[a][2 * b2 + bb];
                if (has_bias)
                    v += bias4[a];
                if (relu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        v[e] = v[e] < 0.0f ? 0.0f : v[e];       // NaN stays NaN
                }
                const u32x2 pk = {KIND == KIND_F16 ? pack_f16x2(v[0], v[1]) : pack_bf16x2(v[0], v[1]),
                                  KIND == KIND_F16 ? pack_f16x2(v[2], v[3]) : pack_bf16x2(v[2], v[3])};
                *(LDS_AS u32x2 *)(stage_h + row * 136 + col * 2) = pk;
            });
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = i * 64 + lane;
                const int row = idx >> 3, c8 = idx & 7;
                // 136-byte pitch keeps rows 8-byte aligned only: two 64-bit reads
                const u32x2 lo = *(LDS_AS u32x2 *)(stage_h + row * 136 + c8 * 16);
                const u32x2 hi = *(LDS_AS u32x2 *)(stage_h + row * 136 + c8 * 16 + 8);
                // non-temporal: C is not read again by this kernel, and lines that do not linger
                // in L2 are not left for the write-back at the end of the kernel (4096^3: -1.4 us)
                if (m0 + wm * PP_WM + b2 * 32 + row < p.M)
                    __builtin_nontemporal_store(u32x4{lo[0], lo[1], hi[0], hi[1]},
                                                (u32x4 *)(crow + (int64_t)(b2 * 32 + row) * p.epi.ldc + c8 * 8));
            }
            __builtin_amdgcn_wave_barrier();
        });
        return;
    }
    static_for<0, PP_TM / 2>([&](auto bc) {
        constexpr int b2 = decltype(bc)::value;
        asm volatile("" ::: "memory");
        static_for<0, 2 * PP_TN>([&](auto aq) {
            constexpr int bb = decltype(aq)::value / PP_TN, a = decltype(aq)::value % PP_TN;
            *(LDS_AS f32x4 *)(stage_f + (16 * bb + (lane & 15)) * PP_EPI_LD + 16 * a + 4 * (lane >> 4)) =
                acc[a][2 * b2 + bb];
        });
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll 2
        for (int i = 0; i < 8; ++i) {
            const int idx = i * 64 + lane;
            const int row = idx >> 4, c4 = idx & 15;
            const f32x4 v = *(LDS_AS f32x4 *)(stage_f + row * PP_EPI_LD + c4 * 4);
            const int64_t m = m0 + wm * PP_WM + b2 * 32 + row;
            const int64_t n = n0 + wn * PP_WN + c4 * 4;
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

// HAS_OFF: the batch-reduce form (tile offsets in device memory) is a kernel of its own, so
// that the plain GEMM kernel carries none of its state or code.
template <bool A_KMAJ, int B_LAY, int KIND, bool HAS_OFF>
__global__ void __launch_bounds__(512)
bf16_pingpong_kernel(Bf16Args p)
{
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    LDS_AS char *smem = (LDS_AS char *)smem_generic;
    select_matrix(p);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Tile offsets live in device memory; a misaligned one sends the whole workgroup
    // to the register-staged loader (2-byte loads).  The vote goes through the dynamic
    // LDS: all 160 KiB are claimed by the slots, so nothing here may use static LDS.
    bool direct = true;
    if constexpr (HAS_OFF) {
        int bad = 0;
        for (int i = tid; i < (int)p.batch; i += 512)
            bad |= (((p.A_off[i] | p.B_off[i]) & 7) != 0);
        const bool wave_bad = __builtin_amdgcn_ballot_w64(bad != 0) != 0;
        LDS_AS int *vote = (LDS_AS int *)smem;
        if (lane == 0)
            vote[w] = wave_bad ? 1 : 0;
        __syncthreads();
        int any_bad = 0;
#pragma unroll
        for (int i = 0; i < PP_NW; ++i)
            any_bad |= vote[i];
        direct = any_bad == 0;
        __syncthreads();
    }
    // Does this wave's operand tile overhang the matrix?  (waves 4-7 load A, 0-3 load B)
    int tm, tn;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const bool edge = (w >> 2) ? ((int64_t)(tm + 1) * PP_BM > p.M)
                               : (B_LAY != LAY_PACKED && (int64_t)(tn + 1) * PP_BN > p.N);
    if constexpr (!HAS_OFF) {
        if (!edge) pp_body<A_KMAJ, B_LAY, true, false, KIND, false>(p);
        else pp_body<A_KMAJ, B_LAY, true, true, KIND, false>(p);
    } else {
        if (direct) {
            if (!edge) pp_body<A_KMAJ, B_LAY, true, false, KIND, true>(p);
            else pp_body<A_KMAJ, B_LAY, true, true, KIND, true>(p);
        } else {
            if (!edge) pp_body<A_KMAJ, B_LAY, false, false, KIND, true>(p);
            else pp_body<A_KMAJ, B_LAY, false, true, KIND, true>(p);
        }
    }
}

// Launch one instance (grid, dynamic LDS, the one-time raise of its LDS limit).
inline hipError_t pingpong_launch(void (*kern)(Bf16Args), const Problem &p)
{
    Bf16Args a;
    fill_common_args(a, p);
    a.tiles_m = (int)((p.M + PP_BM - 1) / PP_BM);
    a.tiles_n = (int)((p.N + PP_BN - 1) / PP_BN);
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)p.split, (unsigned)p.nmat);
    const size_t lds = (size_t)PP_SLOTS * PP_SLOT;
    static thread_local const void *configured[48] = {nullptr};
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
    hipLaunchKernelGGL(kern, grid, dim3(512), lds, p.stream, a);
    return hipGetLastError();
}

// The instances live in three translation units (plain 16-bit GEMM, 16-bit batch-reduce
// with tile offsets, one-byte operands), which build side by side.
hipError_t launch_pingpong_offsets(const Problem &p);
hipError_t launch_pingpong_bytes(const Problem &p);

// Which instance: A k- or m-contiguous, B k-contiguous, n-contiguous or packed.
#define BRG_PP_PICK(kern, p, KIND, OFF)                                                      \
    do {                                                                                     \
        const bool ak_ = (p).transA == 0;                                                    \
        const int lay_ = (p).b_packed ? LAY_PACKED : ((p).transB == 1 ? LAY_K : LAY_MN);     \
        if (ak_ && lay_ == LAY_K) kern = bf16_pingpong_kernel<true, LAY_K, KIND, OFF>;       \
        else if (ak_ && lay_ == LAY_MN) kern = bf16_pingpong_kernel<true, LAY_MN, KIND, OFF>; \
        else if (ak_) kern = bf16_pingpong_kernel<true, LAY_PACKED, KIND, OFF>;              \
        else if (lay_ == LAY_K) kern = bf16_pingpong_kernel<false, LAY_K, KIND, OFF>;        \
        else if (lay_ == LAY_MN) kern = bf16_pingpong_kernel<false, LAY_MN, KIND, OFF>;      \
        else kern = bf16_pingpong_kernel<false, LAY_PACKED, KIND, OFF>;                      \
    } while (0)
#define BRG_PP_PICK_UNPACKED(kern, p, KIND, OFF)                                             \
    do {                                                                                     \
        const bool ak_ = (p).transA == 0, bk_ = (p).transB == 1;                             \
        if (ak_ && bk_) kern = bf16_pingpong_kernel<true, LAY_K, KIND, OFF>;                 \
        else if (ak_) kern = bf16_pingpong_kernel<true, LAY_MN, KIND, OFF>;                  \
        else if (bk_) kern = bf16_pingpong_kernel<false, LAY_K, KIND, OFF>;                  \
        else kern = bf16_pingpong_kernel<false, LAY_MN, KIND, OFF>;                          \
    } while (0)

}  // namespace brg
