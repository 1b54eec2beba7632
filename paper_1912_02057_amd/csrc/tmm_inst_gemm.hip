// k_tmm instantiations: the GEMM (int8 operands, all tile configurations).
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<false, 0, 0>(int, TmmParams&, hipStream_t);
}
