// f32 bulk kernels over a list of chunks (slow to compile: a unit of their own).
#define HFR_HEAVY_TU_LIST
#include "hfr_launch.hip.h"

namespace hfr {

hipError_t launch_reduce_list_f32(const hfr_bucket* items, size_t count, int K, const LaunchShape& sh,
                                 hipStream_t stream) {
    return launch_reduce_bulk_list<F32Traits>(items, count, K, sh, stream);
}

}  // namespace hfr
