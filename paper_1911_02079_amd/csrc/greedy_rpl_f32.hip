// Row-per-lane greedy kernels for binary32 tables.
#include "greedy_rpl_inst.h"

namespace e4q {
hipError_t launch_greedy_rpl_f32(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    return dispatch_greedy_rpl<float>(a, dim, stream);
}
hipError_t launch_greedy_rpl_group_f32(const GreedyGroup& g, int32_t dim, hipStream_t stream)
{
    return dispatch_greedy_rpl_group<float>(g, dim, stream);
}
}  // namespace e4q
