// f32 bulk kernels for more than twelve inputs (slow to compile: a unit of their own).
#define HFR_HEAVY_TU_MANY
#include "hfr_launch.hip.h"

namespace hfr {

template hipError_t launch_reduce_bulk_many<F32Traits>(const void* const* in, int K, void* out, size_t n,
                                                const LaunchShape& sh, hipStream_t stream);

}  // namespace hfr
