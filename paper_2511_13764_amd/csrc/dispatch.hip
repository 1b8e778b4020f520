// Variant table, eligibility rules and the automatic plan.
#include "../../include/brgemm.h"
#include "variants.hpp"

namespace brg {

const char *variant_name(int v)
{
    switch (v) {
    case V_GENERIC: return "generic_64x64x16_f32mfma";
    case V_BF16_128x128: return "bf16_128x128x64";
    case V_BF16_PP256: return "bf16_pingpong_256x256x64";
    case V_F32_128x128: return "f32_128x128x32";
    case V_BF16_STREAM32: return "bf16_stream_32x128x64";
    case V_BF16_STREAM64: return "bf16_stream_64x128x64";
    case V_BF16_STREAM128: return "bf16_stream_128x128x64";
    default: return "";
    }
}

bool variant_eligible(int v, const Problem &p)
{
    switch (v) {
    case V_GENERIC: return true;
    case V_BF16_128x128: return bf16_mfma_eligible(p) && !p.in_f8;      // no 32x32 FP8 form here
    case V_BF16_PP256: return bf16_pingpong_eligible(p);
    case V_F32_128x128: return f32_mfma_eligible(p);
    case V_BF16_STREAM32: return bf16_stream_eligible(p, 32);
    case V_BF16_STREAM64: return bf16_stream_eligible(p, 64);
    case V_BF16_STREAM128: return bf16_stream_eligible(p, 128);
    default: return false;
    }
}

static size_t split_bytes(const Problem &p, int split)
{
    return split > 1 ? (size_t)split * (size_t)p.M * (size_t)p.N * sizeof(float) : 0;
}

// Reduction split for a grid of 128x128 tiles that cannot fill the chip (skinny M,
// small squares, batch-reduce into a small C).  A rough time model, in microseconds,
// with constants fitted to split sweeps on MI355X: a 128x128x64 k-block costs ~0.57 us
// per workgroup, 512 workgroups run at once (two per CU), streaming the operands cannot
// beat ~8 TB/s (they sit in the Infinity Cache when a call repeats), and the fixed-order reduction moves split*M*N*8 bytes at ~3 TB/s plus
// a second launch.
static int split_for_small_grid(const Problem &p, size_t workspace_bytes)
{
    const double tiles = (double)((p.M + 127) / 128) * (double)((p.N + 127) / 128);
    const double kblocks = (double)p.batch * (double)(p.K / 64);
    const double operand_bytes = 2.0 * ((double)p.M + (double)p.N) * (double)p.K * (double)p.batch;
    static const int candidates[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    int best = 1;
    double best_t = 1e30;
    for (int s : candidates) {
        if (s > kMaxSplit || (s > 1 && kblocks / s < 2.0))
            continue;
        if (s > 1 && (size_t)s * (size_t)p.M * (size_t)p.N * sizeof(float) > workspace_bytes)
            continue;
        const double rounds = (double)(int64_t)((tiles * s + 511.0) / 512.0);
        double t_main = rounds * (kblocks / s) * 0.57;
        const double t_stream = operand_bytes / 8.0e6;
        if (t_main < t_stream)
            t_main = t_stream;
        const double t_reduce = s > 1 ? 4.0 + (double)s * (double)p.M * (double)p.N * 8.0 / 3.0e6 : 0.0;
        const double t = 6.0 + t_main + t_reduce;
        if (t < best_t * 0.97) {     // prefer the smaller split on near ties
            best_t = t;
            best = s;
        }
    }
    return best;
}

// Reduction split for the skinny-M streaming kernels (BM x 128 tiles).  Split sweeps
// on the MLP shapes show the time following rounds * (k-blocks per workgroup), where
// rounds = workgroups / 256 rounded up (a CU works through its workgroups at a fixed
// rate), plus a cost per split for the partial tiles that grows with BM.
static int split_for_stream(const Problem &p, int bm, size_t workspace_bytes)
{
    const int64_t tiles = ((p.M + bm - 1) / bm) * ((p.N + 127) / 128);
    const int64_t kblocks = p.batch * (p.K / 64);
    const double per_split = 0.75 * bm / 32.0;
    int best = 1;
    double best_cost = 1e30;
    for (int s = 1; s <= kMaxSplit; ++s) {
        const int64_t per = (kblocks + s - 1) / s;
        if (s > 1 && (per < 8 || split_bytes(p, s) > workspace_bytes))
            continue;
        const double rounds = (double)((tiles * s + 255) / 256);
        const double cost = rounds * (double)per + per_split * s;
        if (cost < best_cost) {
            best_cost = cost;
            best = s;
        }
    }
    return best;
}

// Tile height and reduction split for a grid of at most 256 tiles of 128 x 128 (small
// squares, batch-reduce into a small C): operands that sit in L2 / the Infinity Cache, so
// what counts is how many CUs have work and what a k-block costs a workgroup.  Shorter
// tiles put more workgroups on the chip (1024^3: 256 tiles of 32 x 128 take 9.3 us, 64
// tiles of 128 x 128 take 12.4), as long as they still all run at once; two workgroups of
// the 32- and 64-row kernels share a CU.  Time model in microseconds, constants from
// sweeps over 512^3 ... 2048^3, 512 x 512 x 4096 and the scattered batch-reduce
// configuration: a k-block costs a workgroup 0.20 / 0.29 / 0.42 us at 32 / 64 / 128 rows
// (twice that for a batch-reduce over scattered tiles, where every 64-deep block is a new tile
// somewhere else in memory), a split
// costs a second launch (4.5 us) plus writing and reading its partial tiles.
static void plan_small_grid(const Problem &p, size_t workspace_bytes, bool may_split, int *bm_out, int *split_out)
{
    static const int heights[] = {128, 64, 32};
    static const double block_us[] = {0.42, 0.29, 0.20};
    const int64_t kblocks = p.batch * (p.K / 64);
    double best_t = 1e30;
    *bm_out = 128;
    *split_out = 1;
    // A B operand far larger than the L2s (4 MiB per XCD) is streamed, and every further
    // row of tiles streams it again: then only the tallest tile is considered (measured:
    // 256 x 4096 x 4096 takes 19.0 us as 128-row tiles with split 3 and 24.6 us as 32-row
    // tiles; 1024 x 2048 x 8192 39.8 against 48.9 us with 64-row tiles).
    const bool b_streams = (double)p.N * (double)p.K * (double)p.batch * 2.0 > 8.0 * 1024 * 1024 && p.M > 128;
    for (int i = 0; i < 3; ++i) {
        const int bm = heights[i];
        if (!bf16_stream_eligible(p, bm) || (bm < 128 && p.in_f8))
            continue;
        if (bm < 128 && b_streams && bf16_stream_eligible(p, 128))
            continue;
        const int64_t tiles = ((p.M + bm - 1) / bm) * ((p.N + 127) / 128) * p.nmat;
        if (bm < 128 && tiles > 256)
            continue;
        const int64_t at_once = bm == 128 ? 256 : 512;
        for (int s = 1; s <= (may_split ? kMaxSplit : 1); ++s) {
            const int64_t per = (kblocks + s - 1) / s;
            if (s > 1 && (per < 2 || split_bytes(p, s) > workspace_bytes))
                continue;
            const double rounds = (double)((tiles * s + at_once - 1) / at_once);
            double t = rounds * (double)per * block_us[i] * (p.A_off ? 2.0 : 1.0);
            if (s > 1)
                t += 4.5 + (double)s * (double)p.M * (double)p.N * 4.0 / 4.0e6;
            if (t < best_t * 0.97) {     // near ties: the taller tile, the smaller split
                best_t = t;
                *bm_out = bm;
                *split_out = s;
            }
        }
    }
}

// Reduction split for the fp32 kernel when its 128x128 tiles cannot fill the chip.
// Time model in microseconds, fitted to split sweeps (256^3 ... 2048^3 and the skinny
// MLP shape): one workgroup per CU works through a 128x128x32 k-block in ~2.0 us
// (the fp32 MFMA rate), a launch costs ~8 us of latency, and the reduction adds a
// second launch plus split*M*N*8 bytes at ~3 TB/s.
// Between 257 and 512 tiles of 128 x 128: either the two-stage 128 x 128 kernel with two
// workgroups per CU (about 1.0 us per k-block when all 512 are there) or the 256 x 256
// kernel on a quarter as many tiles with the reduction split so that they fill the chip
// (1.22 us per k-block, plus the partial tiles: split * M * N * 4 bytes read and the
// result written at ~5 TB/s, plus a second launch).  Measured: 2048 x 4096 x 11008 takes
// 174 us the first way and 144 us the second (split 2), 1024 x 8192 x 8192 131 against
// 113 us; at K = 4096 the two are level.  Returns the split for the 256 x 256 kernel, or 0
// to stay with the 128 x 128 kernel.
static int split_for_mid_grid(const Problem &p, size_t workspace_bytes)
{
    if (!bf16_pingpong_eligible(p))
        return 0;
    const double kblocks = (double)p.batch * (double)(p.K / 64);
    const int64_t pp_tiles = ((p.M + 255) / 256) * ((p.N + 255) / 256);
    const double t_128 = 3.0 + kblocks * 1.0;
    int best = 0;
    double best_t = t_128 * 0.92;                   // switch only for a clear gain
    for (int s = 2; s <= kMaxSplit; ++s) {
        if (pp_tiles * s > 256 || kblocks / s < 16.0 || split_bytes(p, s) > workspace_bytes)
            continue;
        const double per = (double)(int64_t)((kblocks + s - 1) / s);
        const double mn = (double)p.M * (double)p.N;
        const double t = 12.0 + per * 1.22 + 4.0 + (s * mn * 4.0 + mn * 2.0) / 5.0e6;
        if (t < best_t) {
            best_t = t;
            best = s;
        }
    }
    return best;
}

static int split_for_f32(const Problem &p, size_t workspace_bytes)
{
    const int64_t tiles = ((p.M + 127) / 128) * ((p.N + 127) / 128);
    const int64_t kblocks = p.K / 32;
    int best = 1;
    double best_t = 1e30;
    for (int s = 1; s <= kMaxSplit; ++s) {
        if (s > 1 && (kblocks / s < 1 || split_bytes(p, s) > workspace_bytes))
            continue;
        const double rounds = (double)((tiles * s + 255) / 256);
        const double per = (double)((kblocks + s - 1) / s);
        const double t_reduce = s > 1 ? 4.0 + (double)s * (double)p.M * (double)p.N * 8.0 / 3.0e6 : 0.0;
        const double t = 8.0 + rounds * per * 2.0 + t_reduce;
        if (t < best_t * 0.97) {
            best_t = t;
            best = s;
        }
    }
    return best;
}

int choose_plan(const Problem &p, size_t workspace_bytes, int forced_variant, int forced_split, Plan *out)
{
    Plan plan{V_GENERIC, 1};
    // A batched call (nmat matrices) multiplies the tile count and never splits.
    const bool single = p.nmat == 1 && !p.in_s8;     // int8 sums are not split (the reduction adds floats)
    const int skinny_bm = p.M <= 32 ? 32 : p.M <= 64 ? 64 : 128;
    if (p.M <= 128 && bf16_stream_eligible(p, skinny_bm)) {
        // Few rows of A: the time goes into streaming B once.
        plan.variant = skinny_bm == 32 ? V_BF16_STREAM32 : skinny_bm == 64 ? V_BF16_STREAM64 : V_BF16_STREAM128;
        plan.split = single ? split_for_stream(p, skinny_bm, workspace_bytes) : 1;
    } else if (bf16_mfma_eligible(p)) {
        // 128x128 tiles while all of them are resident at once (two workgroups per CU:
        // 512), 256x256 tiles beyond that (measured crossover on squares: 2816 -> 3072).
        const int64_t t128 = ((p.M + 127) / 128) * ((p.N + 127) / 128) * p.nmat;
        if (t128 > 512) {
            plan.variant = V_BF16_PP256;
        } else {
            // Up to 256 tiles leave at most one workgroup per CU: a streaming kernel, its
            // tile height by how many workgroups that puts on the chip; between 257 and 512
            // tiles the two-stage kernel wins because two of its workgroups share a CU.
            if (t128 <= 256 && bf16_stream_eligible(p, 128)) {
                int bm = 128, split = 1;
                plan_small_grid(p, workspace_bytes, single, &bm, &split);
                plan.variant = bm == 32 ? V_BF16_STREAM32 : bm == 64 ? V_BF16_STREAM64 : V_BF16_STREAM128;
                plan.split = split;
            } else {
                const int pp_split = (single && !p.in_f8) ? split_for_mid_grid(p, workspace_bytes) : 0;
                if (pp_split > 0) {
                    plan.variant = V_BF16_PP256;
                    plan.split = pp_split;
                } else {
                    plan.variant = (p.in_f8 && bf16_stream_eligible(p, 128)) ? V_BF16_STREAM128 : V_BF16_128x128;
                    plan.split = single ? split_for_small_grid(p, workspace_bytes) : 1;
                }
            }
        }
    }
    if (f32_mfma_eligible(p)) {
        plan.variant = V_F32_128x128;
        plan.split = single ? split_for_f32(p, workspace_bytes) : 1;
    }
    if (forced_variant >= 0) {
        if (forced_variant >= V_COUNT || !variant_eligible(forced_variant, p))
            return BRGEMM_INVALID_ARG;
        plan.variant = forced_variant;
    }
    if (forced_split > 1 && !single)
        return BRGEMM_INVALID_ARG;
    if (forced_split > 0) {
        plan.split = forced_split;
        if (split_bytes(p, plan.split) > workspace_bytes)
            return BRGEMM_WORKSPACE_TOO_SMALL;
    }
    *out = plan;
    return BRGEMM_OK;
}

hipError_t launch_variant(int v, const Problem &p)
{
    switch (v) {
    case V_GENERIC: return p.in_s8 ? launch_generic_s8(p) : launch_generic(p);
    case V_BF16_128x128: return launch_bf16_128x128(p);
    case V_BF16_PP256: return launch_bf16_pingpong(p);
    case V_F32_128x128: return launch_f32_128x128(p);
    case V_BF16_STREAM32: return launch_bf16_stream(p, 32);
    case V_BF16_STREAM64: return launch_bf16_stream(p, 64);
    case V_BF16_STREAM128: return launch_bf16_stream(p, 128);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace brg
