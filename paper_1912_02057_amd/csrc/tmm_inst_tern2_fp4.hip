// k_tmm instantiations: the conv on FP4 (E2M1) codes with the block-tail epilogue.
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<true, 2, 2>(int, TmmParams&, hipStream_t);
}
