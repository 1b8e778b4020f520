// Instances of the 256 x 256 x 64 ping-pong kernel for one-byte operands (int8, FP8 E4M3
// and E5M2; Section 5(c): further packed types through the same kernels), a k-block
// being 128 one-byte k.  Operands contiguous in k use the 2-byte image unchanged; those
// contiguous in m or n go through the one-byte image and ds_read_b64_tr_b8.
#include "bf16_pingpong.hpp"

namespace brg {

hipError_t launch_pingpong_bytes(const Problem &p)
{
    void (*kern)(Bf16Args) = nullptr;
    if (p.in_s8)
        BRG_PP_PICK_UNPACKED(kern, p, KIND_S8, false);
    else if (p.f8_e5m2)
        BRG_PP_PICK_UNPACKED(kern, p, KIND_BF8, false);
    else
        BRG_PP_PICK_UNPACKED(kern, p, KIND_F8, false);
    return pingpong_launch(kern, p);
}

}  // namespace brg
