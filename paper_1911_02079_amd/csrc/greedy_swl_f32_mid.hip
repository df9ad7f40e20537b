// Sub-wave greedy kernels, 32 or 64 elements per lane, float tables.
#define E4Q_SWL_LAYOUTS \
    E4Q_SWL(32, 1) E4Q_SWL(32, 2) E4Q_SWL(32, 4) E4Q_SWL(32, 8) E4Q_SWL(32, 16) E4Q_SWL(32, 32) E4Q_SWL(32, 64) \
    E4Q_SWL(64, 1) E4Q_SWL(64, 2) E4Q_SWL(64, 4) E4Q_SWL(64, 8) E4Q_SWL(64, 16) E4Q_SWL(64, 32) E4Q_SWL(64, 64)
#include "greedy_swl.h"

namespace e4q {
hipError_t launch_greedy_swl_f32_mid(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream)
{
    return dispatch_greedy_swl<float>(a, dim, E, L, stream);
}
}  // namespace e4q
