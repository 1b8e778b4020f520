// Variant table, eligibility rules and the automatic plan.
#include "../../include/brgemm.h"
#include "variants.hpp"

namespace brg {

const char *variant_name(int v)
{
    switch (v) {
    case V_GENERIC: return "generic_64x64x16_f32mfma";
    case V_BF16_256x256: return "bf16_256x256x64";
    case V_BF16_128x128: return "bf16_128x128x64";
    case V_BF16_PP256: return "bf16_pingpong_256x256x64";
    case V_F32_128x128: return "f32_128x128x32";
    default: return "";
    }
}

bool variant_eligible(int v, const Problem &p)
{
    switch (v) {
    case V_GENERIC: return true;
    case V_BF16_256x256:
    case V_BF16_128x128: return bf16_mfma_eligible(p);
    case V_BF16_PP256: return bf16_pingpong_eligible(p);
    case V_F32_128x128: return f32_mfma_eligible(p);
    default: return false;
    }
}

static size_t split_bytes(const Problem &p, int split)
{
    return split > 1 ? (size_t)split * (size_t)p.M * (size_t)p.N * sizeof(float) : 0;
}

int choose_plan(const Problem &p, size_t workspace_bytes, int forced_variant, int forced_split, Plan *out)
{
    Plan plan{V_GENERIC, 1};
    if (bf16_mfma_eligible(p)) {
        // 256x256 tiles once they can occupy most of the 256 CUs, else 128x128.
        const int64_t t256 = ((p.M + 255) / 256) * ((p.N + 255) / 256);
        if (t256 >= 160)
            plan.variant = bf16_pingpong_eligible(p) ? V_BF16_PP256 : V_BF16_256x256;
        else
            plan.variant = V_BF16_128x128;
    }
    if (f32_mfma_eligible(p))
        plan.variant = V_F32_128x128;
    if (forced_variant >= 0) {
        if (forced_variant >= V_COUNT || !variant_eligible(forced_variant, p))
            return BRGEMM_INVALID_ARG;
        plan.variant = forced_variant;
    }
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
    case V_GENERIC: return launch_generic(p);
    case V_BF16_256x256: return launch_bf16_256x256(p);
    case V_BF16_128x128: return launch_bf16_128x128(p);
    case V_BF16_PP256: return launch_bf16_pingpong(p);
    case V_F32_128x128: return launch_f32_128x128(p);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace brg
