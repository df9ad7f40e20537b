// Register-resident 16-means kernels for _Float16 tables.
#include "kmeans16.h"

namespace e4q {
bool launch_kmeans16_rpl_f16(const KMeansArgs& a, int32_t dim, hipStream_t stream)
{
    return launch_kmeans16_rpl<_Float16>(a, dim, stream);
}
}  // namespace e4q
