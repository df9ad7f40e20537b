// Sub-wave greedy kernels, 8 or 16 elements per lane, float tables.
#define E4Q_SWL_LAYOUTS \
    E4Q_SWL(8, 1) E4Q_SWL(8, 2) E4Q_SWL(8, 4) E4Q_SWL(8, 8) E4Q_SWL(8, 16) E4Q_SWL(8, 32) E4Q_SWL(8, 64) \
    E4Q_SWL(16, 1) E4Q_SWL(16, 2) E4Q_SWL(16, 4) E4Q_SWL(16, 8) E4Q_SWL(16, 16) E4Q_SWL(16, 32) E4Q_SWL(16, 64)
#define E4Q_SWL_TWIN_LAYOUTS \
    E4Q_SWL_TWIN(8, 1) E4Q_SWL_TWIN(8, 2) E4Q_SWL_TWIN(8, 4) E4Q_SWL_TWIN(8, 8) E4Q_SWL_TWIN(8, 16) E4Q_SWL_TWIN(8, 32) \
    E4Q_SWL_TWIN(16, 1) E4Q_SWL_TWIN(16, 2) E4Q_SWL_TWIN(16, 4) E4Q_SWL_TWIN(16, 8) E4Q_SWL_TWIN(16, 16) E4Q_SWL_TWIN(16, 32)
#include "greedy_swl.h"

namespace e4q {
hipError_t launch_greedy_swl_f32_small(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream)
{
    return dispatch_greedy_swl<float>(a, dim, E, L, stream);
}
hipError_t launch_greedy_swl_twin_f32(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream)
{
    return dispatch_greedy_swl_twin<float>(a, dim, E, L, stream);
}
}  // namespace e4q
