// e5m2 skewed bulk kernels for eight and nine inputs (slow to compile: a unit of their own).
#define HFR_HEAVY_TU_SKEWED
#include "hfr_launch.hip.h"

namespace hfr {

template hipError_t launch_reduce_bulk_skewed<E5M2Traits>(const void* const* in, int K, void* out, size_t n,
                                                  const LaunchShape& sh, hipStream_t stream);

}  // namespace hfr
