// k_tmm instantiations: the GEMM on FP4 (E2M1) codes.
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<false, 0, 2>(int, TmmParams&, hipStream_t);
}
