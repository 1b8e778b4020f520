// Instances of the 256 x 256 x 64 ping-pong kernel for batch-reduce calls whose tiles are
// given by offset lists (Section 2.1: the tiles of one call need not be contiguous).
#include "bf16_pingpong.hpp"

namespace brg {

hipError_t launch_pingpong_offsets(const Problem &p)
{
    void (*kern)(Bf16Args) = nullptr;
    if (p.in_f16)
        BRG_PP_PICK(kern, p, KIND_F16, true);
    else
        BRG_PP_PICK(kern, p, KIND_BF16, true);
    return pingpong_launch(kern, p);
}

}  // namespace brg
