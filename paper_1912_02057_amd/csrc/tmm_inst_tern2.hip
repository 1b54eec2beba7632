// k_tmm instantiations: the conv with the block-tail epilogue.
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<true, 2, 0>(int, TmmParams&, hipStream_t);
}
