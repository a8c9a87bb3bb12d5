// Host-side plumbing shared by the translation units of libhfr (not installed).
#pragma once

#include <hip/hip_runtime_api.h>
#include <stddef.h>

#include <atomic>

#include "../../include/hfr.h"

namespace hfr {

// Launch shape of one kernel call, decided on the host.
struct LaunchShape {
    bool bulk;       // lock-step shape with deferred store bursts (large inputs)
    int unroll;      // wide shape: 16-byte vectors per lane per trip: 1, 2 or 4
    bool aligned16;  // every pointer is 16-byte aligned
    unsigned grid;   // workgroups
    int epilogue;    // K-way sum only: 0 plain sum, 1 multiply the fp32 sum by `scale`,
                     // 2 the last input is the remote partial (combine, then scale)
    float scale;
    int skew;        // bulk K-way sum: stream skew pattern 0..3 (0 = none)
    int block;       // bulk K-way sum: lanes per workgroup (a multiple of 32; 0 = 256)
    int pace;        // bulk K-way sum: pause after each trip, in units of 64 clocks
    int wgs_per_cu;  // wide K-way sum: most workgroups resident on a compute unit (0 = no limit)
};

constexpr int kBlock = 256;  // lanes per workgroup: four wave64

// Knobs (hfr_set_tuning / environment); 0 or -1 mean "library default".
// Atomic: another thread may turn a knob while a launch reads it.
struct Tuning {
    std::atomic<long> grid_cap{0};
    std::atomic<long> unroll{0};
    std::atomic<long> bulk_grid{0};
    std::atomic<long> bulk_min_bytes{0};
    std::atomic<long> bulk_skew{0};
    std::atomic<long> bucket_fold{0};
    std::atomic<long> placement_online{0};
    std::atomic<long> segment_mib{0};
    std::atomic<long> bulk_block{0};
    std::atomic<long> bulk_pace{0};
    std::atomic<long> wide_wgs_per_cu{0};
    std::atomic<long> bucket_list{0};
};
const Tuning& tuning();
Tuning& tuning_mut();

// Compute units of the current device (cached per device).
hipError_t device_cu_count(int* cus);

// Host decision of the launch shape for n elements of elem_size bytes and
// `streams` read/write streams per element (K inputs, or 2 for the combine).
hipError_t choose_shape(size_t n, size_t elem_size, int n_inputs, bool aligned16, LaunchShape* shape);

// Default bound on the workgroups of a wide or batched launch that share a
// compute unit (0 = none), by input count and bytes per buffer.
int default_wide_wgs_per_cu(int n_inputs, size_t bytes_per_buffer);

// Kernel launchers, one translation unit per element type.
hipError_t launch_reduce_sum_f32(const void* const* in, int K, void* out, size_t n,
                                 const LaunchShape& sh, hipStream_t stream);
hipError_t launch_reduce_sum_bf16(const void* const* in, int K, void* out, size_t n,
                                  const LaunchShape& sh, hipStream_t stream);
hipError_t launch_reduce_sum_f16(const void* const* in, int K, void* out, size_t n,
                                 const LaunchShape& sh, hipStream_t stream);
hipError_t launch_combine_avg_f16(const void* a, const void* b, void* out, size_t n, float scale,
                                  const LaunchShape& sh, hipStream_t stream);
hipError_t launch_combine_avg_f32(const void* a, const void* b, void* out, size_t n, float scale,
                                  const LaunchShape& sh, hipStream_t stream);
hipError_t launch_combine_avg_bf16(const void* a, const void* b, void* out, size_t n, float scale,
                                   const LaunchShape& sh, hipStream_t stream);

// Batched launch of `count` small buckets; count must not exceed batch_capacity(K).
hipError_t launch_reduce_batched_f32(const hfr_bucket* buckets, size_t count, int K, bool aligned16,
                                     hipStream_t stream);
hipError_t launch_reduce_batched_bf16(const hfr_bucket* buckets, size_t count, int K, bool aligned16,
                                      hipStream_t stream);
hipError_t launch_reduce_batched_f16(const hfr_bucket* buckets, size_t count, int K, bool aligned16,
                                     hipStream_t stream);

#define HFR_DECLARE_DTYPE_LAUNCHERS(sfx)                                                                   \
    hipError_t launch_reduce_sum_##sfx(const void* const* in, int K, void* out, size_t n,                  \
                                       const LaunchShape& sh, hipStream_t stream);                         \
    hipError_t launch_combine_avg_##sfx(const void* a, const void* b, void* out, size_t n, float scale,   \
                                        const LaunchShape& sh, hipStream_t stream);                        \
    hipError_t launch_reduce_batched_##sfx(const hfr_bucket* buckets, size_t count, int K, bool aligned16, \
                                           hipStream_t stream);
HFR_DECLARE_DTYPE_LAUNCHERS(e4m3)
HFR_DECLARE_DTYPE_LAUNCHERS(e5m2)
#undef HFR_DECLARE_DTYPE_LAUNCHERS

// K-way sum over a chunk table in DEVICE memory (entries laid out as hfr_chunk).
hipError_t launch_reduce_table_f32(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                   hipStream_t stream);
hipError_t launch_reduce_table_bf16(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                    hipStream_t stream);
hipError_t launch_reduce_table_f16(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                   hipStream_t stream);
hipError_t launch_reduce_table_e4m3(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                    hipStream_t stream);
hipError_t launch_reduce_table_e5m2(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                    hipStream_t stream);

// One bulk-shape launch over a list of chunks that lie apart (K = 8 or 16, 16-byte aligned buffers);
// count must not exceed list_capacity(K); sh carries the grid, the workgroup size and the pause.
#define HFR_DECLARE_LIST_LAUNCHER(sfx)                                                                    \
    hipError_t launch_reduce_list_##sfx(const hfr_bucket* items, size_t count, int K, const LaunchShape& sh, \
                                        hipStream_t stream);
HFR_DECLARE_LIST_LAUNCHER(f32)
HFR_DECLARE_LIST_LAUNCHER(bf16)
HFR_DECLARE_LIST_LAUNCHER(f16)
HFR_DECLARE_LIST_LAUNCHER(e4m3)
HFR_DECLARE_LIST_LAUNCHER(e5m2)
#undef HFR_DECLARE_LIST_LAUNCHER
// Entries per list launch: what fits the 4 KiB kernel-argument segment ((K + 4) eight-byte words each).
inline size_t list_capacity(int K) { return (3840 - 16) / (size_t(K + 4) * 8); }
inline bool list_available(int K) { return K == 8 || K == 16; }

// Broadcast: nbytes from src to each of the K destinations.
hipError_t launch_broadcast(const void* src, void* const* dst, int K, size_t nbytes, bool aligned16,
                            hipStream_t stream);

// The launchers of one element type.
struct DtypeOps {
    hipError_t (*reduce)(const void* const*, int, void*, size_t, const LaunchShape&, hipStream_t);
    hipError_t (*combine)(const void*, const void*, void*, size_t, float, const LaunchShape&, hipStream_t);
    hipError_t (*batched)(const hfr_bucket*, size_t, int, bool, hipStream_t);
    hipError_t (*table)(const void*, size_t, size_t, int, hipStream_t);
    hipError_t (*list)(const hfr_bucket*, size_t, int, const LaunchShape&, hipStream_t);
};
const DtypeOps* dtype_ops(hfr_dtype dt);  // nullptr for an unknown code

// Buckets per batched launch: what fits the 4 KiB kernel-argument segment
// ((K + 3) eight-byte words per bucket, 3824 bytes of table).
inline size_t batch_capacity(int K) { return (3840 - 16) / (size_t(K + 3) * 8); }
// Largest bucket (bytes per buffer) that is folded into a batched launch.
constexpr size_t kBatchMaxBytes = size_t(8) << 20;

// Records the text of a failed HIP call for hfr_last_error() and maps it.
hfr_status fail_hip(hipError_t e, const char* what);
// Records `text` for hfr_last_error() and returns `status`.
hfr_status fail_text(hfr_status status, const char* text);

// Argument validation (host only, touches no HIP state).
size_t dtype_size(hfr_dtype dt);  // 0 for an unknown code
hfr_status validate_reduce(const void* const* in, int K, const void* out, size_t n, hfr_dtype dt);

// Enqueue one validated K-way sum (shared by hfr_reduce_sum and the bucket scheduler).
// skew: -1 = the knob's / the recorded pattern for this placement, 0..3 = that pattern.
hfr_status enqueue_reduce(const void* const* in, int K, void* out, size_t n, hfr_dtype dt,
                          hipStream_t stream, int epilogue = 0, float scale = 1.0f, int skew = -1);
// Whether a K-way sum of n elements would take the bulk shape (it then occupies
// every compute unit on its own).
hfr_status reduce_is_bulk(int K, size_t n, hfr_dtype dt, bool* bulk);
hfr_status list_shape(int K, hfr_dtype dt, int skew, LaunchShape* sh);  // skew 0 or 3; sh->grid == 0: no bulk shape (knob)

// Skew patterns of the bulk K-way sum, keyed by how the K input buffers and the
// output lie relative to each other (distances from input 0 in 4 KiB units:
// chunks, slices and launch segments of the same buffers share a key), found by
// hfr_tune_placement or by trial launches on the fly.
constexpr int kSkewChoices = 4;  // patterns 0..3 of the bulk kernel
unsigned skew_mask(int K, int epilogue);  // bit p: pattern p of the bulk kernel exists
bool skew_applies(int K, bool aligned16, int epilogue);
void placement_store(const void* const* in, int K, const void* out, size_t elem_size, int skew);
void placement_clear();  // also destroys the events of unfinished measurements
// 0 = unknown placement, 1 = being measured, 2 = recorded (then *skew is the pattern)
int placement_query(const void* const* in, int K, const void* out, size_t elem_size, int* skew);
// One bulk launch whose skew pattern comes from the table (see hfr_api.cpp).
hipError_t launch_by_placement(const void* const* in, int K, void* out, size_t n, hfr_dtype dt, LaunchShape sh,
                               hipStream_t stream);

// Static chunk table of hfr_reduce_chunks_noalloc: looks up its device address
// for the current device (once per device). table may be nullptr.
struct ChunkDesc;
hfr_status noalloc_setup(ChunkDesc** table);

// Worker-stream pool of the current device.
struct StreamPool;
// pool_acquire makes sure of n_streams worker streams and returns with the pool
// LOCKED (one fork/join sequence at a time per device); pool_unlock releases it.
hfr_status pool_acquire(int n_streams, StreamPool** pool);
hipStream_t pool_stream(StreamPool* pool, int w);
hipEvent_t pool_fork_event(StreamPool* pool);
hipEvent_t pool_join_event(StreamPool* pool, int w);
void pool_unlock(StreamPool* pool);
hfr_status pool_destroy_all();

}  // namespace hfr
