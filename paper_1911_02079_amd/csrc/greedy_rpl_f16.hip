// Row-per-lane greedy kernels for binary16 tables (rows are widened to binary32 once, in registers).
#include "greedy_rpl_inst.h"

namespace e4q {
hipError_t launch_greedy_rpl_f16(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    return dispatch_greedy_rpl<_Float16>(a, dim, stream);
}
hipError_t launch_greedy_rpl_group_f16(const GreedyGroup& g, int32_t dim, hipStream_t stream)
{
    return dispatch_greedy_rpl_group<_Float16>(g, dim, stream);
}
}  // namespace e4q
