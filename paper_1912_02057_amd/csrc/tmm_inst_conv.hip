// k_tmm instantiations: the conv with the plain epilogue.
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<true, 0, 0>(int, TmmParams&, hipStream_t);
}
