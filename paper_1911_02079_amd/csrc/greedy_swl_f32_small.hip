// Sub-wave greedy kernels, short chunks per lane (8 to 64 elements), float tables.
#define E4Q_SWL_LAYOUTS                                                                          \
    E4Q_SWL(8, 1) E4Q_SWL(8, 2) E4Q_SWL(8, 4) E4Q_SWL(8, 8) E4Q_SWL(8, 16) E4Q_SWL(8, 32) E4Q_SWL(8, 64) \
    E4Q_SWL(16, 1) E4Q_SWL(16, 64) E4Q_SWL(32, 1) E4Q_SWL(32, 2) E4Q_SWL(32, 4) E4Q_SWL(32, 8)            \
    E4Q_SWL(32, 16) E4Q_SWL(32, 32) E4Q_SWL(32, 64) E4Q_SWL(64, 1) E4Q_SWL(64, 64)
#include "greedy_swl.h"

namespace e4q {
hipError_t launch_greedy_swl_f32_small(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream)
{
    return dispatch_greedy_swl<float>(a, dim, E, L, stream);
}
}  // namespace e4q
