// f32 bulk kernels with skew pattern 3 for the input counts other than eight and nine
// (slow to compile: a unit of their own).
#define HFR_HEAVY_TU_SKEWED3
#include "hfr_launch.hip.h"

namespace hfr {

template hipError_t launch_reduce_bulk_skewed3<F32Traits>(const void* const* in, int K, void* out, size_t n,
                                                   const LaunchShape& sh, hipStream_t stream);

}  // namespace hfr
