// Register-resident 16-means kernels for float tables.
#include "kmeans16.h"

namespace e4q {
bool launch_kmeans16_rpl_f32(const KMeansArgs& a, int32_t dim, hipStream_t stream)
{
    return launch_kmeans16_rpl<float>(a, dim, stream);
}
}  // namespace e4q
