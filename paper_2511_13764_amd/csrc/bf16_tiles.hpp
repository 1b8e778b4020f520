// Building blocks shared by the tuned bf16 kernels: LDS tile images and their
// swizzles, MFMA fragment reads, the XCD-aware tile order and the 4-column epilogue.
#pragma once
#include "common.hpp"
#include "variants.hpp"
#include <type_traits>

namespace brg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;

// The matrix instruction per operand kind.  Fragments travel as 16-byte registers
// (bf16x8) whatever they hold; for int8 the same 16 bytes are 16 k-values, the
// instruction contracts 64 (resp. 32) of them per step and the accumulators hold
// int32 bit patterns in the same registers.
template <int KIND>
__device__ __forceinline__ f32x4 mfma_16x16x32(bf16x8 a, bf16x8 b, f32x4 c)
{
    if constexpr (KIND == KIND_F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else if constexpr (KIND == KIND_S8)
        return __builtin_bit_cast(f32x4, __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                                            __builtin_bit_cast(i32x4, c), 0, 0, 0));
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
template <int KIND>
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c)
{
    if constexpr (KIND == KIND_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else if constexpr (KIND == KIND_S8)
        return __builtin_bit_cast(f32x16, __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b),
                                                                             __builtin_bit_cast(i32x16, c), 0, 0, 0));
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

typedef __attribute__((ext_vector_type(8))) int i32x8;

// FP8 (both operands E4M3, or both E5M2): v_mfma_f32_16x16x128_f8f6f4 contracts 128 k
// per instruction, 32 bytes per lane and operand, given here as the two 16-byte chunks a
// lane read.  Which k-bytes sit where inside the 32 is irrelevant as long as both
// operands agree.  The two format fields of the instruction take 0 for E4M3, 1 for E5M2.
template <int KIND>
__device__ __forceinline__ f32x4 mfma_16x16x128_f8(bf16x8 a_lo, bf16x8 a_hi, bf16x8 b_lo, bf16x8 b_hi, f32x4 c)
{
    const i32x8 a = __builtin_shufflevector(__builtin_bit_cast(i32x4, a_lo), __builtin_bit_cast(i32x4, a_hi), 0, 1, 2, 3, 4, 5, 6, 7);
    const i32x8 b = __builtin_shufflevector(__builtin_bit_cast(i32x4, b_lo), __builtin_bit_cast(i32x4, b_hi), 0, 1, 2, 3, 4, 5, 6, 7);
    constexpr int FMT = KIND == KIND_BF8 ? 1 : 0;
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, FMT, FMT, 0, 0, 0, 0);
}

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

constexpr int BK = 64;                  // k-block depth (elements) = 128 bytes of bf16

struct Bf16Args {
    int64_t M, N, K, batch;
    const uint16_t *A;
    const int64_t *A_off;
    int64_t lda;
    const uint16_t *B;
    const int64_t *B_off;
    int64_t ldb;
    Epilogue epi;
    int split;
    float *partial;
    int tiles_m, tiles_n;
    int64_t ms_a, ms_b, ms_c;       // element strides between the matrices of a batched call (blockIdx.z)
};

// Batched matmul: point the arguments at matrix blockIdx.z.
__device__ __forceinline__ void select_matrix(Bf16Args &p)
{
    const int64_t z = blockIdx.z;
    p.A += z * p.ms_a;
    p.B += z * p.ms_b;
    p.epi.C = (char *)p.epi.C + z * p.ms_c * (p.epi.c_f32 ? 4 : 2);
}

// Host side: fill the fields every bf16 launcher shares.
inline void fill_common_args(Bf16Args &a, const Problem &p)
{
    // The kernels address their operands in 2-byte units along k; a problem with
    // one-byte elements (both operands k-contiguous) is handed over with K and the leading
    // dimensions halved.
    const int64_t u = in_8bit(p) ? 2 : 1;
    a.M = p.M; a.N = p.N; a.K = p.K / u; a.batch = p.batch;
    a.A = (const uint16_t *)p.A; a.A_off = p.A_off; a.lda = p.lda / u;
    a.B = (const uint16_t *)p.B; a.B_off = p.B_off; a.ldb = p.ldb / u;
    a.epi.beta = p.beta; a.epi.C = p.C; a.epi.ldc = p.ldc; a.epi.c_f32 = p.c_f32; a.epi.c_f16 = p.in_f16;
    a.epi.c_i32 = p.in_s8;
    a.epi.bias = p.bias; a.epi.relu = p.relu;
    a.split = p.split; a.partial = p.partial;
    a.ms_a = p.ms_a; a.ms_b = p.ms_b; a.ms_c = p.ms_c;
}

// s_waitcnt immediates for gfx9-family encodings: vmcnt in bits [3:0] and [15:14],
// expcnt [6:4], lgkmcnt [11:8].
__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }
__device__ __forceinline__ void wait_vmcnt8() { __builtin_amdgcn_s_waitcnt(0x0F78); }
// Wait until at most N vector-memory loads of this wave are outstanding (N <= 63).
template <int N>
__device__ __forceinline__ void wait_vmcnt_le()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Workgroup barrier that neither the compiler's scheduler nor its memory-operation
// motion may cross.  Unlike __syncthreads() it emits no wait of its own: callers wait
// for exactly the loads and LDS reads that must be complete.
__device__ __forceinline__ void block_sync()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Tell the compiler a pointer is wave-uniform (keeps it in SGPRs).
__device__ __forceinline__ const uint16_t *uniform_ptr(const uint16_t *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const uint16_t *)(((uint64_t)hi << 32) | lo);
}

// Tile offsets of a batch-reduce call (Section 2.1: the tiles of one call need not be
// contiguous), 64 at a time in two registers of the wave: lane l holds the offset of
// tile `base + l`, and a wave-uniform tile index is served by v_readlane.  With
// 64-deep tiles every k-block starts a new tile; fetched one by one from memory, each
// offset is a dependent global load in front of that block's loads.  Here that
// latency is paid once per 64 tiles.
struct TileOffsets {
    const int64_t *off;
    int last;               // batch - 1
    int base;
    uint32_t lo, hi;

    __device__ __forceinline__ void refill(int first, int lane)
    {
        const int i = first + lane < last ? first + lane : last;
        const uint64_t v = (uint64_t)off[i];
        lo = (uint32_t)v;
        hi = (uint32_t)(v >> 32);
        // Make the load complete here, inside the rare refill path.  Otherwise the compiler, which
        // must assume at the join that this load may still be pending, puts an s_waitcnt vmcnt(0) in
        // front of every v_readlane of get() - and vmcnt also counts the global->LDS loads in
        // flight, so every tile switch would drain the whole prefetch pipeline (measured: +0.3 us
        // per 64-deep tile).  The empty statement uses and redefines both registers.
        asm volatile("" : "+v"(lo), "+v"(hi));
        base = first;
    }
    __device__ __forceinline__ void init(const int64_t *offsets, int64_t batch, int first, int lane)
    {
        off = offsets;
        last = (int)batch - 1;
        refill(first, lane);
    }
    // i: wave-uniform tile index, base <= i < batch.
    __device__ __forceinline__ int64_t get(int i, int lane)
    {
        if (i - base >= 64)
            refill(i, lane);
        const int l = i - base;
        const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)lo, l);
        const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)hi, l);
        return (int64_t)(((uint64_t)b << 32) | a);
    }
};

// The same load in its scalar-base form: a wave-uniform 64-bit base in SGPRs plus
// a 32-bit per-lane byte offset.  With 64-bit per-lane addresses the load's
// address read competes with the MFMAs of the other wave on the SIMD for register
// file bandwidth and issue takes ~2.5x longer (measured); this form does not.
// lds_addr is the wave-uniform LDS byte address (goes to M0).  The statement carries
// no "memory" clobber on purpose: with one, the compiler drains vmcnt and lgkmcnt
// before every load.  It is therefore invisible to the compiler's wait-count
// insertion and may be moved across ordinary LDS reads; callers wait on vmcnt
// themselves and fence with volatile asm / barriers where order matters.
__device__ __forceinline__ void load16_to_lds_saddr(const char *base, uint32_t lane_off, uint32_t lds_addr)
{
    // readfirstlane: the "s" constraint alone does not move a value the compiler
    // believes divergent into SGPRs (it is free when the value already is uniform).
    const uint64_t b = (uint64_t)base;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const uint64_t ub = ((uint64_t)hi << 32) | lo;
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(la), "v"(lane_off), "s"(ub)
                 : "m0");
}

// ---------------------------------------------------------------------------
// Operand tile whose contiguous direction is k ("K-major": A with transA == 0,
// B with transB == 1).  LDS image: row r (an m or n index) takes 128 bytes; its
// 16-byte chunk c (8 consecutive k) sits at chunk position c ^ ((r >> 1) & 7).
// The LDS has 64 banks of 4 bytes, so two rows share one 256-byte bank window and
// the 16 rows a 128-bit read serves per clock must land on 16 different 16-byte
// positions of it: rows of equal parity need 8 different XOR values, hence r >> 1.
// ---------------------------------------------------------------------------
template <int ROWS, int NW>
struct KMajorTile {
    static constexpr int kInstr = ROWS / 8;          // wave-instructions per tile
    static constexpr int kPerWave = kInstr / NW;

    __device__ static uint32_t dst_byte(int w, int j) { return (uint32_t)(w * kPerWave + j) * 1024u; }
    // What this lane fetches for wave-instruction j of wave w, as a 32-bit byte offset
    // from the tile origin (row row0, first k of the block): lets the load use a uniform
    // base + lane offset.  row_limit redirects rows past a ragged edge to a valid row.
    __device__ static uint32_t src_rel_bytes(int w, int j, int lane, int64_t row0, int64_t row_limit, int64_t ld)
    {
        const int g = w * kPerWave + j;
        int64_t row = row0 + 8 * g + (lane >> 3);
        row = row < row_limit ? row : row_limit - 1;
        const int c = (lane & 7) ^ (((8 * g + (lane >> 3)) >> 1) & 7);
        return (uint32_t)(((row - row0) * ld + 8 * c) * 2);
    }

    // Scalar-base form of the same addressing.  Wave-instruction g of the tile reads
    // rows 8g..8g+7: a per-instruction scalar offset g * instr_stride_bytes(ld), plus a
    // lane offset that depends on g only through its parity (the swizzle term 4*(g&1)).
    // Lanes whose row lies outside the matrix are switched off instead of redirected.
    __device__ static int64_t instr_stride_bytes(int64_t ld) { return 8 * ld * 2; }
    __device__ static int64_t instr_offset_bytes(int g, int64_t ld) { return (int64_t)g * 8 * ld * 2; }
    // Element offset of the tile's first row, and of one k-block step, in the matrix.
    __device__ static int64_t origin(int64_t first, int64_t ld) { return first * ld; }
    __device__ static int64_t kstep(int64_t) { return BK; }
    __device__ static uint32_t lane_off_bytes(int parity, int lane, int64_t ld)
    {
        const int c = (lane & 7) ^ ((4 * parity + (lane >> 4)) & 7);
        return (uint32_t)(((int64_t)(lane >> 3) * ld + 8 * c) * 2);
    }
    __device__ static int32_t lane_delta_bytes(int) { return 0; }
    __device__ static bool delta_applies(int) { return false; }
    __device__ static bool lane_valid(int g, int lane, int64_t row0, int64_t row_limit)
    {
        return row0 + 8 * g + (lane >> 3) < row_limit;
    }

    // Byte offset of the 8 k-values lane `lane` needs for MFMA tile `t` (32 rows) and
    // k-slice ks (16 k): row t*32 + lane%32, chunk 2*ks + lane/32.
    __device__ static uint32_t frag_byte(int row_base, int t, int ks, int lane)
    {
        const int r = row_base + t * 32 + (lane & 31);
        const int c = 2 * ks + (lane >> 5);
        return (uint32_t)(r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
    }
    __device__ static bf16x8 read_frag(LDS_AS char *tile, int row_base, int t, int ks, int lane)
    {
        return *(LDS_AS bf16x8 *)(tile + frag_byte(row_base, t, ks, lane));
    }
    // Operand of v_mfma_f32_16x16x32_bf16 for 16-row tile t and 32-deep k-step s: lane l
    // holds row t*16 + l%16 and the 8 k-values of chunk 4*s + l/16.  The 128-deep FP8
    // instruction takes 32 bytes per lane: reads s = 0 and s = 1 of the same tile, i.e.
    // chunks l/16 and 4 + l/16 of the row (which k-bytes a lane holds is free as long as
    // both operands agree; the adjacent pair 2*(l/16), 2*(l/16) + 1 costs about 4
    // bank-conflict cycles per read with this swizzle, this pair none).
    __device__ static bf16x8 read_frag16(LDS_AS char *tile, int row_base, int t, int s, int lane)
    {
        const int r = row_base + t * 16 + (lane & 15);
        const int c = 4 * s + (lane >> 4);
        return *(LDS_AS bf16x8 *)(tile + (uint32_t)(r * 128 + ((c ^ ((r >> 1) & 7)) << 4)));
    }
};

// ---------------------------------------------------------------------------
// Operand tile whose contiguous direction is m or n ("MN-major": A with
// transA == 1, B with transB == 0).  LDS image: k-row kr takes COLS*2 bytes; its
// 16-byte chunk c (8 consecutive m/n) sits at chunk position c ^ swz(kr) with
// swz(kr) = ((kr & 3) << 2) | (((kr >> 3) & 1) << 1).  The first term spreads the
// four k-rows one transposing read touches over distinct banks; the second keeps
// k-rows kr and kr + 8, which the two 16-lane blocks of a half-wave read for the
// 16x16x32 MFMA operand, 32 bytes apart.
// ---------------------------------------------------------------------------
template <int COLS, int NW>
struct MNMajorTile {
    static constexpr int kChunksPerRow = COLS / 8;
    static constexpr int kRowBytes = COLS * 2;
    static constexpr int kInstr = BK * kChunksPerRow / 64;
    static constexpr int kPerWave = kInstr / NW;

    __device__ static int swz(int kr) { return ((kr & 3) << 2) | (((kr >> 3) & 1) << 1); }

    __device__ static uint32_t dst_byte(int w, int j) { return (uint32_t)(w * kPerWave + j) * 1024u; }
    __device__ static uint32_t src_rel_bytes(int w, int j, int lane, int64_t col0, int64_t col_limit, int64_t ld)
    {
        const int idx = (w * kPerWave + j) * 64 + lane;
        const int kr = idx / kChunksPerRow;
        const int pc = idx % kChunksPerRow;
        const int c = pc ^ swz(kr);
        const int64_t rel = (col0 + 8 * c < col_limit) ? 8 * c : 0;
        return (uint32_t)(((int64_t)kr * ld + rel) * 2);
    }

    // Scalar-base form: wave-load g covers 2 (256-column tile) or 4 (128) k-rows.  The
    // lane offset depends on g through its parity (first swizzle term, 256 columns
    // only) and through bit 3 of its k-rows (second term), which moves the chunk by
    // +-32 bytes: offset = lane_off_bytes(g & 1) + (delta_applies(g) ? lane_delta_bytes : 0).
    __device__ static int64_t instr_offset_bytes(int g, int64_t ld) { return (int64_t)g * (64 / kChunksPerRow) * ld * 2; }
    __device__ static int64_t origin(int64_t first, int64_t) { return first; }
    __device__ static int64_t kstep(int64_t ld) { return (int64_t)BK * ld; }
    __device__ static uint32_t lane_off_bytes(int parity, int lane, int64_t ld)
    {
        static_assert(kChunksPerRow == 32 || kChunksPerRow == 16, "row of 256 or 128 elements");
        const int kr_in = lane / kChunksPerRow;
        const int pc = lane % kChunksPerRow;
        const int c = pc ^ ((((64 / kChunksPerRow) * parity + kr_in) & 3) << 2);
        return (uint32_t)(((int64_t)kr_in * ld + 8 * c) * 2);
    }
    __device__ static int32_t lane_delta_bytes(int lane) { return ((lane % kChunksPerRow) & 2) ? -32 : 32; }
    __device__ static bool delta_applies(int g) { return (((64 / kChunksPerRow) * g) >> 3) & 1; }
    __device__ static bool lane_valid(int g, int lane, int64_t col0, int64_t col_limit)
    {
        const int kr = (64 / kChunksPerRow) * g + lane / kChunksPerRow;
        const int c = (lane % kChunksPerRow) ^ swz(kr);
        return col0 + 8 * c < col_limit;
    }

    // ds_read_b64_tr_b16 works on blocks of 16 lanes: lane i of a block supplies the
    // address of 4 consecutive columns (4*(i%4)..) of k-row (i/4) and receives, for
    // column i, the 4 k-values of those rows.  Two reads give the 8 k-values of the
    // MFMA operand: k = 8*(lane/32) + 4*rd + 0..3 within the 16-deep slice.
    __device__ static bf16x8 read_frag(LDS_AS char *tile, int col_base, int t, int ks, int lane)
    {
        const int b = lane >> 4, i = lane & 15;
        const int col = col_base + t * 32 + 16 * (b & 1) + 4 * (i & 3);
        const int c = col >> 3;
        const int within = (col & 7) * 2;
        s16x4 v[2];
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            const int kr = ks * 16 + 8 * (b >> 1) + 4 * rd + (i >> 2);
            const uint32_t byte = (uint32_t)(kr * kRowBytes + ((c ^ swz(kr)) << 4) + within);
            v[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + byte));
        }
        s16x8 r = __builtin_shufflevector(v[0], v[1], 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, r);
    }
    // Operand of v_mfma_f32_16x16x32_bf16 for 16-column tile t and 32-deep k-step s:
    // block b of 16 lanes holds k = 8*b .. 8*b+7 of the step for column t*16 + lane%16,
    // i.e. two transposing reads of k-rows 32*s + 8*b + 4*rd + 0..3.
    __device__ static bf16x8 read_frag16(LDS_AS char *tile, int col_base, int t, int s, int lane)
    {
        const int b = lane >> 4, i = lane & 15;
        const int col = col_base + t * 16 + 4 * (i & 3);
        const int c = col >> 3;
        const int within = (col & 7) * 2;
        s16x4 v[2];
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            const int kr = s * 32 + 8 * b + 4 * rd + (i >> 2);
            const uint32_t byte = (uint32_t)(kr * kRowBytes + ((c ^ swz(kr)) << 4) + within);
            v[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(tile + byte));
        }
        s16x8 r = __builtin_shufflevector(v[0], v[1], 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, r);
    }
};

// ---------------------------------------------------------------------------
// The same for one-byte elements (int8, FP8): an operand whose contiguous direction
// is m or n.  A k-block is 128 k-rows of COLS bytes (the kernels count k in 2-byte
// units, so their 64-deep block is 128 one-byte k).  LDS image: k-row kr takes COLS
// bytes; its 16-byte chunk c (16 consecutive m/n) sits at chunk position c ^ swz(kr).
// ds_read_b64_tr_b8 works on blocks of 16 lanes: lane i of a block supplies the
// address of 8 consecutive columns (8*(i%2)..) of k-row i/2 and receives, for column
// i, the 8 k-values of those rows in k order.  The 16 k-values a lane needs per
// matrix instruction (k = 64*s + 16*(lane/16) + 0..15 for the 16x16 forms: the same
// bytes a k-contiguous operand's 16-byte read gives it) are two such reads.  A
// half-wave thus reads one chunk column of 16 k-rows kr0 + 0..7 and kr0 + 16 + 0..7:
// the swizzle gives those 16 rows 16 different 16-byte positions of a 256-byte bank
// window (256-byte rows: three bits of kr and bit 4; 128-byte rows hold two k-rows
// per window, so bits 1-2 of kr and bit 4).
// ---------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(2))) int i32x2;

template <int COLS, int NW>
struct MNMajorTile8 {
    static_assert(COLS == 256 || COLS == 128, "row of 256 or 128 one-byte elements");
    static constexpr int kChunksPerRow = COLS / 16;
    static constexpr int kRowBytes = COLS;
    static constexpr int kRowsPerInstr = 1024 / COLS;               // k-rows one wave-load covers
    static constexpr int kInstr = 2 * BK * COLS / 1024;
    static constexpr int kPerWave = kInstr / NW;

    __device__ static int swz(int kr)
    {
        return COLS == 256 ? ((kr & 7) | (((kr >> 4) & 1) << 3)) : (((kr >> 1) & 3) | (((kr >> 4) & 1) << 2));
    }

    // `ld` is the row pitch in 2-byte units (the host halves the leading dimensions of
    // one-byte operands), offsets returned are bytes.
    __device__ static uint32_t dst_byte(int w, int j) { return (uint32_t)(w * kPerWave + j) * 1024u; }
    __device__ static uint32_t src_rel_bytes(int w, int j, int lane, int64_t col0, int64_t col_limit, int64_t ld)
    {
        const int idx = (w * kPerWave + j) * 64 + lane;
        const int kr = idx / kChunksPerRow;
        const int pc = idx % kChunksPerRow;
        const int c = pc ^ swz(kr);
        const int64_t rel = (col0 + 16 * c < col_limit) ? 16 * c : 0;
        return (uint32_t)((int64_t)kr * ld * 2 + rel);
    }

    __device__ static int64_t origin(int64_t first, int64_t) { return first / 2; }
    __device__ static int64_t kstep(int64_t ld) { return 2 * (int64_t)BK * ld; }
    // Scalar-base form (256-byte rows only): wave-load g covers k-rows 4g + lane / 16.  The
    // swizzle depends on g through its parity (bits 0-2 of the k-row) and through bit 2
    // (bit 4 of the k-row), which moves the chunk by +-128 bytes:
    // offset = lane_off_bytes(g & 1) + (delta_applies(g) ? lane_delta_bytes : 0).
    __device__ static int64_t instr_offset_bytes(int g, int64_t ld) { return (int64_t)g * kRowsPerInstr * ld * 2; }
    __device__ static uint32_t lane_off_bytes(int parity, int lane, int64_t ld)
    {
        static_assert(COLS == 256, "scalar-base addressing is written for 256-byte rows");
        const int kr_in = lane / kChunksPerRow;
        const int pc = lane % kChunksPerRow;
        const int c = pc ^ ((4 * parity + kr_in) & 7);
        return (uint32_t)((int64_t)kr_in * ld * 2 + 16 * c);
    }
    __device__ static int32_t lane_delta_bytes(int lane) { return ((lane % kChunksPerRow) & 8) ? -128 : 128; }
    __device__ static bool delta_applies(int g) { return (g >> 2) & 1; }
    __device__ static bool lane_valid(int g, int lane, int64_t col0, int64_t col_limit)
    {
        const int kr = kRowsPerInstr * g + lane / kChunksPerRow;
        const int c = (lane % kChunksPerRow) ^ swz(kr);
        return col0 + 16 * c < col_limit;
    }

    // 16 k-values from k-row kr0 on for the 16 columns from col on (col % 16 == 0), lane
    // i of each 16-lane block receiving column col + i.
    __device__ static bf16x8 read16(LDS_AS char *tile, int col, int kr0, int i)
    {
        const int c = col >> 4;
        i32x2 v[2];
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            const int kr = kr0 + 8 * rd + (i >> 1);
            const uint32_t byte = (uint32_t)(kr * kRowBytes + ((c ^ swz(kr)) << 4) + 8 * (i & 1));
            v[rd] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2 *)(tile + byte));
        }
        const i32x4 r = __builtin_shufflevector(v[0], v[1], 0, 1, 2, 3);
        return __builtin_bit_cast(bf16x8, r);
    }
    // Operand of the 32x32 int8 instruction for 32-column tile t and 32-deep k-slice ks:
    // lane l holds column t*32 + l%32 and k = 32*ks + 16*(l/32) + 0..15.
    __device__ static bf16x8 read_frag(LDS_AS char *tile, int col_base, int t, int ks, int lane)
    {
        const int b = lane >> 4;
        return read16(tile, col_base + t * 32 + 16 * (b & 1), 32 * ks + 16 * (b >> 1), lane & 15);
    }
    // Operand of the 16x16 instructions for 16-column tile t and 64-deep k-step s.
    __device__ static bf16x8 read_frag16(LDS_AS char *tile, int col_base, int t, int s, int lane)
    {
        return read16(tile, col_base + t * 16, 64 * s + 16 * (lane >> 4), lane & 15);
    }
};

// ---------------------------------------------------------------------------
// B operand packed ahead of time in groups of 8 consecutive k: the VNNI layout of
// Section 2.2 / Figure 1 with a factor of 8, the 8 bf16 values one MFMA lane
// consumes.  Element (k, n) sits at ((k / 8) * n_pitch + n) * 8 + k % 8; "ld" is
// the element count of one k-group row, n_pitch * 8.  The packer pads K to a
// multiple of 64 and the column pitch to a multiple of 256 with zeros, so tiles
// never overhang the image.  A k-block of a COLS-wide tile is 8 runs of COLS * 16
// contiguous bytes; the LDS image keeps that order ([k-group][column][16 bytes]),
// global -> LDS is a straight copy, and a fragment read takes 32 consecutive
// 16-byte chunks per half-wave: no swizzle, no bank conflicts, no transposing read.
// ---------------------------------------------------------------------------
template <int COLS, int NW>
struct PackedTile {
    static constexpr int kPerGroup = COLS / 64;             // wave-loads per k-group row
    static constexpr int kInstr = 8 * kPerGroup;
    static constexpr int kPerWave = kInstr / NW;

    __device__ static uint32_t dst_byte(int w, int j) { return (uint32_t)(w * kPerWave + j) * 1024u; }
    __device__ static uint32_t src_rel_bytes(int w, int j, int lane, int64_t, int64_t, int64_t ld)
    {
        const int g = w * kPerWave + j;
        return (uint32_t)(((int64_t)(g / kPerGroup) * ld + (int64_t)(64 * (g % kPerGroup) + lane) * 8) * 2);
    }
    __device__ static int64_t instr_offset_bytes(int g, int64_t ld)
    {
        return ((int64_t)(g / kPerGroup) * ld + (int64_t)(g % kPerGroup) * 512) * 2;
    }
    __device__ static int64_t origin(int64_t first, int64_t) { return first * 8; }
    __device__ static int64_t kstep(int64_t ld) { return 8 * ld; }
    __device__ static uint32_t lane_off_bytes(int, int lane, int64_t) { return (uint32_t)lane * 16u; }
    __device__ static int32_t lane_delta_bytes(int) { return 0; }
    __device__ static bool delta_applies(int) { return false; }
    __device__ static bool lane_valid(int, int, int64_t, int64_t) { return true; }
    __device__ static bf16x8 read_frag(LDS_AS char *tile, int col_base, int t, int ks, int lane)
    {
        const int kg = 2 * ks + (lane >> 5);
        const int col = col_base + t * 32 + (lane & 31);
        return *(LDS_AS bf16x8 *)(tile + (uint32_t)(kg * COLS + col) * 16u);
    }
    __device__ static bf16x8 read_frag16(LDS_AS char *tile, int col_base, int t, int s, int lane)
    {
        const int kg = 4 * s + (lane >> 4);
        const int col = col_base + t * 16 + (lane & 15);
        return *(LDS_AS bf16x8 *)(tile + (uint32_t)(kg * COLS + col) * 16u);
    }
};

// Operand layouts as template arguments (a bool "k-major" converts to the first two).
constexpr int LAY_MN = 0, LAY_K = 1, LAY_PACKED = 2;
// KIND selects the one-byte image for an m/n-contiguous operand; k-contiguous one-byte
// operands use the 2-byte image as it is (two k per unit).
template <int EXTENT, int NW, int LAYOUT, int KIND = KIND_BF16>
struct TileOf;
template <int EXTENT, int NW, int KIND>
struct TileOf<EXTENT, NW, LAY_K, KIND> { typedef KMajorTile<EXTENT, NW> type; };
template <int EXTENT, int NW, int KIND>
struct TileOf<EXTENT, NW, LAY_MN, KIND> {
    typedef std::conditional_t<kind_is_8bit(KIND), MNMajorTile8<EXTENT, NW>, MNMajorTile<EXTENT, NW>> type;
};
template <int EXTENT, int NW, int KIND>
struct TileOf<EXTENT, NW, LAY_PACKED, KIND> { typedef PackedTile<EXTENT, NW> type; };

// XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs (each with
// its own L2), so workgroup w is renumbered to t = (w % 8) * (T/8) + w / 8: every
// XCD then owns a contiguous run of logical tiles, and logical tiles are walked in
// groups of GM tile-rows so that a run shares few A row-panels and B column-panels.
// Logical tile number t -> (tm, tn): tiles are walked in groups of GM tile-rows, so a
// contiguous run of logical tiles shares few A row-panels and B column-panels.
__device__ __forceinline__ void group_walk(int t, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int GM = 4;
    const int per_group = GM * tiles_n;
    const int group = t / per_group;
    const int first_m = group * GM;
    const int gsize = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
    const int in_group = t - group * per_group;
    tm = first_m + in_group % gsize;
    tn = in_group / gsize;
}

__device__ __forceinline__ void tile_coords(int w, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int T = tiles_m * tiles_n;
    const int T8 = T & ~7;
    int t = w;
    if (w < T8)
        t = (w & 7) * (T8 >> 3) + (w >> 3);
    group_walk(t, tiles_m, tiles_n, tm, tn);
}

// Work assignment of a launch whose grid is (tiles, split): which tile and which slice
// of the reduction this workgroup takes.  Workgroups are dealt to the XCDs round-robin
// in launch order (x fastest), so launch index L is renumbered to
// L' = (L % 8) * (W / 8) + L / 8 and L' is read slice-major: every XCD owns a
// contiguous run of (slice, tile) pairs, i.e. as few reduction slices as possible.
// With a split of 8 each XCD's L2 then holds one eighth of the tiles of a
// batch-reduce call instead of all of them (8 MiB of scattered tiles do not fit one
// 4 MiB L2; fetched by every XCD they made each 64-deep block wait for the
// last-level cache).
__device__ __forceinline__ void slice_major_coords(int tiles, int &tile, int &slice)
{
    const int W = (int)(gridDim.x * gridDim.y);
    const int L = (int)(blockIdx.x + gridDim.x * blockIdx.y);
    const int W8 = W & ~7;
    const int Lp = L < W8 ? (L & 7) * (W8 >> 3) + (L >> 3) : L;
    slice = Lp / tiles;
    tile = Lp - slice * tiles;
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Four consecutive columns n..n+3 of row m, values already final sums.  `left` is
// N - n (columns that exist); `vec` says 16-byte (fp32) / 8-byte (bf16) accesses
// are aligned.
__device__ __forceinline__ void store4_partial(float *dst, int64_t left, bool vec, float v0, float v1, float v2,
                                               float v3)
{
    if (left <= 0)
        return;
    if (vec && left >= 4) {
        *(f32x4 *)dst = f32x4{v0, v1, v2, v3};
    } else {
        dst[0] = v0;
        if (left > 1) dst[1] = v1;
        if (left > 2) dst[2] = v2;
        if (left > 3) dst[3] = v3;
    }
}

__device__ __forceinline__ void store4_epilogue(const Epilogue &e, int64_t m, int64_t n, int64_t left, bool vec,
                                                float v0, float v1, float v2, float v3)
{
    if (left <= 0)
        return;
    if (e.c_i32 && vec && left >= 4) {
        i32x4 r = {__float_as_int(v0), __float_as_int(v1), __float_as_int(v2), __float_as_int(v3)};
        if (e.beta != 0.0f)
            r += *(const i32x4 *)((const int32_t *)e.C + m * e.ldc + n);
        *(i32x4 *)((int32_t *)e.C + m * e.ldc + n) = r;
        return;
    }
    if (!(vec && left >= 4)) {
        epilogue_store(e, v0, m, n);
        if (left > 1) epilogue_store(e, v1, m, n + 1);
        if (left > 2) epilogue_store(e, v2, m, n + 2);
        if (left > 3) epilogue_store(e, v3, m, n + 3);
        return;
    }
    if (e.beta != 0.0f) {
        if (e.c_f32) {
            const f32x4 old = *(const f32x4 *)((const float *)e.C + m * e.ldc + n);
            v0 = fmaf(e.beta, old[0], v0);
            v1 = fmaf(e.beta, old[1], v1);
            v2 = fmaf(e.beta, old[2], v2);
            v3 = fmaf(e.beta, old[3], v3);
        } else {
            const uint2 old = *(const uint2 *)((const uint16_t *)e.C + m * e.ldc + n);
            v0 = fmaf(e.beta, c16_to_f32((uint16_t)old.x, e.c_f16), v0);
            v1 = fmaf(e.beta, c16_to_f32((uint16_t)(old.x >> 16), e.c_f16), v1);
            v2 = fmaf(e.beta, c16_to_f32((uint16_t)old.y, e.c_f16), v2);
            v3 = fmaf(e.beta, c16_to_f32((uint16_t)(old.y >> 16), e.c_f16), v3);
        }
    }
    if (e.bias) {
        // n is a multiple of 4, so the 16-byte read is aligned exactly when the bias
        // pointer is; a bias that starts inside a larger buffer is read by element.
        if ((((uintptr_t)e.bias) & 15) == 0) {
            const f32x4 bv = *(const f32x4 *)(e.bias + n);
            v0 += bv[0]; v1 += bv[1]; v2 += bv[2]; v3 += bv[3];
        } else {
            v0 += e.bias[n]; v1 += e.bias[n + 1]; v2 += e.bias[n + 2]; v3 += e.bias[n + 3];
        }
    }
    if (e.relu) {
        v0 = v0 < 0.0f ? 0.0f : v0;
        v1 = v1 < 0.0f ? 0.0f : v1;
        v2 = v2 < 0.0f ? 0.0f : v2;
        v3 = v3 < 0.0f ? 0.0f : v3;
    }
    if (e.c_f32) {
        *(f32x4 *)((float *)e.C + m * e.ldc + n) = f32x4{v0, v1, v2, v3};
    } else {
        uint2 out;
        out.x = pack_c16x2(v0, v1, e.c_f16);
        out.y = pack_c16x2(v2, v3, e.c_f16);
        *(uint2 *)((uint16_t *)e.C + m * e.ldc + n) = out;
    }
}

// Store one wave's register tile (TN x TM accumulators of 32x32, computed with the
// operands swapped so that lane l owns row l%32 and 4 consecutive columns per group
// of 4 registers): raw fp32 partial sums for a split reduction, else the epilogue.
// m_base / n_base: the row / first column this lane owns in accumulator (0, 0).
template <int TM, int TN>
__device__ __forceinline__ void store_wave_tile(const Bf16Args &p, f32x16 (&acc)[TN][TM], int64_t m_base,
                                                int64_t n_base, int split_index)
{
    if (p.split > 1) {
        float *part = p.partial + (int64_t)split_index * p.M * p.N;
        const bool vec = (p.N & 3) == 0;
        static_for<0, TM>([&](auto bc) {
            constexpr int b = decltype(bc)::value;
            const int64_t m = m_base + b * 32;
            if (m < p.M) {
                static_for<0, TN * 4>([&](auto aq) {
                    constexpr int a = decltype(aq)::value / 4, q = decltype(aq)::value % 4;
                    const int64_t n = n_base + a * 32 + q * 8;
                    store4_partial(part + m * p.N + n, p.N - n, vec, acc[a][b][4 * q + 0], acc[a][b][4 * q + 1],
                                   acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                });
            }
        });
    } else {
        const bool vec = (p.epi.ldc & 3) == 0 && (((uintptr_t)p.epi.C) & 15) == 0;
        static_for<0, TM>([&](auto bc) {
            constexpr int b = decltype(bc)::value;
            const int64_t m = m_base + b * 32;
            if (m < p.M) {
                static_for<0, TN * 4>([&](auto aq) {
                    constexpr int a = decltype(aq)::value / 4, q = decltype(aq)::value % 4;
                    const int64_t n = n_base + a * 32 + q * 8;
                    store4_epilogue(p.epi, m, n, p.N - n, vec, acc[a][b][4 * q + 0], acc[a][b][4 * q + 1],
                                    acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                });
            }
        });
    }
}

// Store one wave's register tile: TN x TM accumulators of 16x16 from
// v_mfma_f32_16x16x32_bf16 with the operands swapped, so that lane l owns row l%16
// and the 4 consecutive columns 4*(l/16) .. +3 of every accumulator.  Raw fp32 partial
// sums for a split reduction, else the epilogue.  m_base / n_base: the row / first
// column this lane owns in accumulator (0, 0).
template <int TM, int TN>
__device__ __forceinline__ void store_wave_tile16(const Bf16Args &p, f32x4 (&acc)[TN][TM], int64_t m_base,
                                                  int64_t n_base, int split_index)
{
    if (p.split > 1) {
        float *part = p.partial + (int64_t)split_index * p.M * p.N;
        const bool vec = (p.N & 3) == 0;
        static_for<0, TM>([&](auto bc) {
            constexpr int b = decltype(bc)::value;
            const int64_t m = m_base + b * 16;
            if (m < p.M) {
                static_for<0, TN>([&](auto ac) {
                    constexpr int a = decltype(ac)::value;
                    const int64_t n = n_base + a * 16;
                    store4_partial(part + m * p.N + n, p.N - n, vec, acc[a][b][0], acc[a][b][1], acc[a][b][2],
                                   acc[a][b][3]);
                });
            }
        });
    } else {
        const bool vec = (p.epi.ldc & 3) == 0 && (((uintptr_t)p.epi.C) & 15) == 0;
        static_for<0, TM>([&](auto bc) {
            constexpr int b = decltype(bc)::value;
            const int64_t m = m_base + b * 16;
            if (m < p.M) {
                static_for<0, TN>([&](auto ac) {
                    constexpr int a = decltype(ac)::value;
                    const int64_t n = n_base + a * 16;
                    store4_epilogue(p.epi, m, n, p.N - n, vec, acc[a][b][0], acc[a][b][1], acc[a][b][2],
                                    acc[a][b][3]);
                });
            }
        });
    }
}

}  // namespace brg
