// Kernel variants and the host-side plan (which variant, how many reduction
// splits).  Tile selection is by hand-tuned rule, as in Section 5(a) of the
// paper (tile sizes are chosen per target by sweeping).
#pragma once
#include "common.hpp"

namespace brg {

enum Variant {
    V_GENERIC = 0,      // any shape / alignment, fp32 MFMA, 64x64 tile
    V_BF16_128x128,     // bf16, 128x128x64 workgroup tile, 64x64 wave tile
    V_BF16_PP256,       // bf16, 256x256x64 tile, 8 waves in alternating memory/compute phases
    V_F32_128x128,      // fp32, 128x128x32 tile, fp32 MFMA
    V_BF16_STREAM32,    // bf16, skinny M: 32x128x64 tile, deep LDS ring (HBM-bound shapes)
    V_BF16_STREAM64,    // bf16, skinny M: 64x128x64 tile, deep LDS ring
    V_BF16_STREAM128,   // bf16, skinny M: 128x128x64 tile, deep LDS ring
    V_COUNT
};

constexpr int kMaxSplit = 16;

struct Plan {
    int variant;
    int split;
};

const char *variant_name(int v);

// Pick variant and split for a validated, non-empty problem.  forced_variant < 0
// and forced_split <= 0 mean automatic.  Returns a BRGEMM_* code.
int choose_plan(const Problem &p, size_t workspace_bytes, int forced_variant, int forced_split, Plan *out);

// True when `v` can run `p` (alignment and layout rules of the tuned kernels).
bool variant_eligible(int v, const Problem &p);

hipError_t launch_variant(int v, const Problem &p);

// bf16_mfma.hip
bool bf16_mfma_eligible(const Problem &p);
hipError_t launch_bf16_128x128(const Problem &p);
// f32_mfma.hip
bool f32_mfma_eligible(const Problem &p);
hipError_t launch_f32_128x128(const Problem &p);
// bf16_pingpong.hip
bool bf16_pingpong_eligible(const Problem &p);
hipError_t launch_bf16_pingpong(const Problem &p);

// bf16_stream.hip
bool bf16_stream_eligible(const Problem &p, int bm);
hipError_t launch_bf16_stream(const Problem &p, int bm);

}  // namespace brg
