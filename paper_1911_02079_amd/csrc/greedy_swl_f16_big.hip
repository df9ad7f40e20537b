// Sub-wave greedy kernels, 128 elements per lane, _Float16 tables.
#define E4Q_SWL_LAYOUTS \
    E4Q_SWL(128, 1) E4Q_SWL(128, 2) E4Q_SWL(128, 4) E4Q_SWL(128, 8) E4Q_SWL(128, 16) E4Q_SWL(128, 32)
#include "greedy_swl.h"

namespace e4q {
hipError_t launch_greedy_swl_f16_big(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream)
{
    return dispatch_greedy_swl<_Float16>(a, dim, E, L, stream);
}
}  // namespace e4q
