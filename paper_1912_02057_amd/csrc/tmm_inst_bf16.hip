// k_tmm instantiations with bf16 operands (the weight-only ternary GEMM / conv).
#include "tmm_kernel.h"

namespace rtn {

hipError_t tmm_launch_bf16(bool conv, int variant, TmmParams& prm, hipStream_t st)
{
    if (conv) {
        switch (variant) {
            case 0: return launch_cfg<64, 64, 2, 2, 4, 4, true, 0, 0, 1>(prm, st);
            case 1: return launch_cfg<128, 128, 2, 2, 3, 2, true, 0, 0, 1>(prm, st);
            case 2: return launch_cfg<128, 256, 2, 2, 2, 2, true, 0, 0, 1>(prm, st);
            case 3: return launch_cfg<64, 256, 1, 4, 2, 3, true, 0, 0, 1>(prm, st);
            default: return hipErrorInvalidValue;
        }
    }
    switch (variant) {
        case 0: return launch_cfg<64, 64, 2, 2, 4, 4, false, 0, 0, 1>(prm, st);
        case 1: return launch_cfg<128, 128, 2, 2, 4, 2, false, 0, 0, 1>(prm, st);
        case 2: return launch_cfg<256, 256, 2, 2, 4, 1, false, 0, 0, 1>(prm, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace rtn
