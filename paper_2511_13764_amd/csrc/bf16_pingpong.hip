// The 256 x 256 x 64 ping-pong kernel (see bf16_pingpong.hpp): its instances for plain
// 16-bit GEMMs, and the entry point that sends batch-reduce calls with tile offsets and
// one-byte operands to the translation units holding theirs.
#include "bf16_pingpong.hpp"

namespace brg {

hipError_t launch_bf16_pingpong(const Problem &p)
{
    if (in_8bit(p))
        return launch_pingpong_bytes(p);
    if (p.A_off)
        return launch_pingpong_offsets(p);
    void (*kern)(Bf16Args) = nullptr;
    if (p.in_f16)
        BRG_PP_PICK(kern, p, KIND_F16, false);
    else
        BRG_PP_PICK(kern, p, KIND_BF16, false);
    return pingpong_launch(kern, p);
}

// Same alignment rules as the 4-wave kernel (which include the 32-bit lane offsets).
bool bf16_pingpong_eligible(const Problem &p) { return bf16_mfma_eligible(p); }

}  // namespace brg
