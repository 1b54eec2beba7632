// k_tmm instantiations: the conv with the ternarizing epilogue.
#include "tmm_dispatch.inc"

namespace rtn {
template hipError_t tmm_launch_index_raw<true, 1, 0>(int, TmmParams&, hipStream_t);
}
