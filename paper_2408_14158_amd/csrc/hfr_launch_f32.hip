// fp32 kernel variants and their launchers.
#include "hfr_launch.hip.h"

namespace hfr {

hipError_t launch_reduce_sum_f32(const void* const* in, int K, void* out, size_t n,
                                 const LaunchShape& sh, hipStream_t stream) {
    return launch_reduce_any_k<F32Traits, 4>(in, K, out, n, sh, stream);
}

hipError_t launch_combine_avg_f32(const void* a, const void* b, void* out, size_t n, float scale,
                                  const LaunchShape& sh, hipStream_t stream) {
    return launch_combine_any<F32Traits, 4>(a, b, out, n, scale, sh, stream);
}

hipError_t launch_reduce_batched_f32(const hfr_bucket* buckets, size_t count, int K, bool aligned16,
                                    hipStream_t stream) {
    return launch_batched_any_k<F32Traits, 4>(buckets, count, K, aligned16, stream);
}

hipError_t launch_reduce_table_f32(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                   hipStream_t stream) {
    return launch_table_any_k<F32Traits, 4>(table, n_chunks, chunk_elems_hint, K, stream);
}

}  // namespace hfr
