// k_tmm instantiations: the conv on FP4 (E2M1) codes with the plain epilogue.
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<true, 0, 2>(int, TmmParams&, hipStream_t);
}
