// Sub-wave greedy kernels with a lane count per row that is not a power of two, float tables.
#define E4Q_SWL_LAYOUTS
#define E4Q_SWL_ANY_E E4Q_SWL_E(8) E4Q_SWL_E(16) E4Q_SWL_E(32) E4Q_SWL_E(64) E4Q_SWL_E(128)
#include "greedy_swl.h"

namespace e4q {
hipError_t launch_greedy_swl_any_f32(const GreedyArgs& a, int32_t dim, int E, int lanes, hipStream_t stream)
{
    return dispatch_greedy_swl_any<float>(a, dim, E, lanes, stream);
}
}  // namespace e4q
