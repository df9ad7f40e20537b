// Register-resident 16-means kernels with a masked tail (dimensions that are not multiples of 8), _Float16 tables.
#include "kmeans16.h"

namespace e4q {
bool launch_kmeans16_rpl_tail_f16(const KMeansArgs& a, int32_t dim, hipStream_t stream)
{
    return launch_kmeans16_rpl_tail<_Float16>(a, dim, stream);
}
}  // namespace e4q
