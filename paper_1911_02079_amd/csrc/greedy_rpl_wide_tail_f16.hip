// Row-per-lane greedy kernels with a masked tail for binary16 tables of dimension 129 .. 223 (not multiples of 8).
#include "greedy_rpl_inst.h"

namespace e4q {
hipError_t launch_greedy_rpl_wide_tail_f16(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    return dispatch_greedy_rpl_wide_tail<_Float16>(a, dim, stream);
}
}  // namespace e4q
