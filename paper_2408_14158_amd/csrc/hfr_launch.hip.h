// Host-side dispatch from runtime (K, unroll, alignment, cache policy) to the
// compile-time kernel variants. Included once per element type so the two
// types compile in parallel.
#pragma once

#include "hfr_internal.h"
#include "hfr_kernels.hip.h"

namespace hfr {

// Largest unroll whose K * U 16-byte loads still fit a register budget that
// keeps at least four waves per SIMD resident (wide shape).
constexpr int max_unroll_for_k(int K) { return K <= 4 ? 4 : (K <= 8 ? 2 : 1); }

// Bulk shape: vectors per lane per trip chosen so that a wave keeps 8 to 16
// loads in flight, and trips per store burst so that a lane parks 32 result
// vectors (128 KiB per workgroup and burst) for every K.
constexpr int bulk_unroll_for_k(int K) { return K == 1 ? 8 : (K == 2 ? 4 : (K <= 4 ? 2 : 1)); }
constexpr int bulk_result_vecs_for_k(int) { return 32; }

// LDS reserved per workgroup so that at most `wgs` workgroups share a compute
// unit (160 KiB each): just over the share that one more workgroup would need.
inline size_t lds_for_wgs_per_cu(int wgs) {
    if (wgs <= 0) return 0;
    const size_t total = size_t(160) << 10;
    const size_t bytes = total / size_t(wgs + 1) + 1024;
    return bytes > (size_t(128) << 10) ? (size_t(128) << 10) : bytes;
}

// sh.epilogue selects the plain sum, the fused average or the fused combine.
template <typename T, int K, int U, int ALIGN>
hipError_t launch_reduce_variant(const void* const* in, void* out, size_t n, const LaunchShape& sh,
                                 hipStream_t stream) {
    PtrPack<K> pack;
    for (int j = 0; j < K; ++j) pack.p[j] = in[j];
    const dim3 grid(sh.grid), block(kBlock);
    const size_t lds = lds_for_wgs_per_cu(sh.wgs_per_cu);
    auto launch = [&](size_t lds_bytes) -> hipError_t {
        if (sh.epilogue == kEpiScale) {
            return launch_kernel_lds(reduce_sum_kernel<T, K, U, kBlock, ALIGN, kEpiScale>, grid, block, lds_bytes, stream, pack, out, n, sh.scale);
        } else if (sh.epilogue == kEpiCombine) {
            if constexpr (K >= 2)
                return launch_kernel_lds(reduce_sum_kernel<T, K, U, kBlock, ALIGN, kEpiCombine>, grid, block, lds_bytes, stream, pack, out, n, sh.scale);
            else
                return hipErrorInvalidValue;
        } else {
            return launch_kernel_lds(reduce_sum_kernel<T, K, U, kBlock, ALIGN, kEpiNone>, grid, block, lds_bytes, stream, pack, out, n, 1.0f);
        }
    };
    hipError_t e = launch(lds);
    if (e != hipSuccess && lds != 0) {
        // a runtime that refuses the reservation: the limit is an optimisation only
        (void)hipGetLastError();
        e = launch(0);
    }
    return e;
}

// Trips per burst of the bulk shape: a workgroup's trips (whole tiles / grid,
// rounded up) split evenly over the fewest bursts of at most R trips.
inline unsigned bulk_trips_per_burst(size_t n, size_t vec_elems, size_t tile_vecs, unsigned grid, unsigned R) {
    const size_t ntiles = n / vec_elems / tile_vecs;
    size_t per_wg = (ntiles + grid - 1) / grid;
    if (per_wg == 0) per_wg = 1;
    const size_t bursts = (per_wg + R - 1) / R;
    return unsigned((per_wg + bursts - 1) / bursts);
}

// The bulk shape needs 16-byte aligned buffers (the host routes anything else
// to the wide shape). Skewed variants: for eight and nine inputs (the per-node
// GPU count of the paper's cluster, and that plus the remote partial) every
// pattern with every epilogue; for the other input counts of the bulk shape
// pattern 3 with the plain sum (the one pattern that repairs every uniform
// stride measured; see skew_mask in the host code).
constexpr bool bulk_skew_available(int K) { return K >= 5 && K <= HFR_MAX_K; }
constexpr bool bulk_skew_every_pattern(int K) { return K == 8 || K == 9; }
// Kernels that take long to compile (template-unrolled trips) live in a
// translation unit of their own per element type: K > 12, and the skewed ones.

// Upper bound of the bulk kernels' workgroup size (their launch bound): up to
// seven inputs the measured optimum needs more than four waves per compute
// unit; from ten inputs on it never does, and those kernels keep the
// register budget of a 256-lane workgroup.
constexpr int bulk_max_block_for_k(int K) { return K <= 7 ? 384 : 256; }
// The plain (not skewed) kernels for eight and nine inputs gain from more
// lanes as well (the fused combine of seven peers and the remote partial most:
// 3 to 11 %) and fit the register budget of a 384-lane workgroup; their skewed
// variants, which hold the leading streams' vectors too, do not.
constexpr int bulk_max_block_for(int K, int skew) {
    return (K == 8 || K == 9) && skew == 0 ? 384 : bulk_max_block_for_k(K);
}

// PLAIN_ONLY: only the kernel of the plain sum is built (any other epilogue is an error).
template <typename T, int K, int SKEW, bool PLAIN_ONLY = false>
hipError_t launch_reduce_bulk_skew(const void* const* in, void* out, size_t n, const LaunchShape& sh,
                                   hipStream_t stream) {
    constexpr int U = bulk_unroll_for_k(K);
    constexpr int R = bulk_result_vecs_for_k(K) / U;
    constexpr int kMaxBlock = bulk_max_block_for(K, SKEW);
    const unsigned max_block = unsigned(kMaxBlock);
    PtrPack<K> pack;
    for (int j = 0; j < K; ++j) pack.p[j] = in[j];
    // whole waves, at least one, at most what the kernel was compiled for
    unsigned lanes = sh.block > 0 ? unsigned(sh.block) : unsigned(kBlock);
    lanes = lanes < 64u ? 64u : (lanes > max_block ? max_block : lanes);
    lanes &= ~31u;
    const dim3 grid(sh.grid), block(lanes);
    const unsigned trips = bulk_trips_per_burst(n, T::kVec, size_t(lanes) * U, sh.grid, R);
    const size_t ntiles = n / T::kVec / (size_t(lanes) * U);  // whole tiles
    const unsigned pace = sh.pace > 0 ? unsigned(sh.pace) : 0u;
    if (sh.epilogue == kEpiScale) {
        if constexpr (!PLAIN_ONLY)
            return launch_kernel(reduce_sum_bulk_kernel<T, K, U, R, kMaxBlock, 16, kEpiScale, SKEW>, grid, block, stream, pack, out, n, ntiles, sh.scale, trips, pace);
        else
            return hipErrorInvalidValue;
    } else if (sh.epilogue == kEpiCombine) {
        if constexpr (K >= 2 && !PLAIN_ONLY)
            return launch_kernel(reduce_sum_bulk_kernel<T, K, U, R, kMaxBlock, 16, kEpiCombine, SKEW>, grid, block, stream, pack, out, n, ntiles, sh.scale, trips, pace);
        else
            return hipErrorInvalidValue;
    } else {
        return launch_kernel(reduce_sum_bulk_kernel<T, K, U, R, kMaxBlock, 16, kEpiNone, SKEW>, grid, block, stream, pack, out, n, ntiles, 1.0f, trips, pace);
    }
}

// Defined (and instantiated for their element type) in the heavy translation
// units: more than twelve inputs, the skewed variants for eight and nine
// inputs, and pattern 3 for the other input counts.
template <typename T>
hipError_t launch_reduce_bulk_many(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                                   hipStream_t stream);
template <typename T>
hipError_t launch_reduce_bulk_skewed(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                                     hipStream_t stream);
template <typename T>
hipError_t launch_reduce_bulk_skewed3(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                                      hipStream_t stream);

// The bulk shape over a list of chunks (K = 8 and 16: the per-node GPU count of
// the paper's cluster and the largest K). Defined in a translation unit of its
// own per element type.
constexpr bool bulk_list_available(int K) { return K == 8 || K == 16; }
template <typename T>
hipError_t launch_reduce_bulk_list(const hfr_bucket* items, size_t count, int K, const LaunchShape& sh,
                                   hipStream_t stream);

#ifdef HFR_HEAVY_TU_LIST
template <typename T, int K, int SKEW>
hipError_t launch_reduce_bulk_list_ks(const hfr_bucket* items, size_t count, const LaunchShape& sh, hipStream_t stream) {
    constexpr int R = bulk_result_vecs_for_k(K);  // one vector per lane and trip
    constexpr int kMaxBlock = bulk_max_block_for(K, SKEW);
    if (count == 0 || count > size_t(list_capacity<K>()) || sh.grid == 0) return hipErrorInvalidValue;
    unsigned lanes = sh.block > 0 ? unsigned(sh.block) : unsigned(kBlock);
    lanes = lanes < 64u ? 64u : (lanes > unsigned(kMaxBlock) ? unsigned(kMaxBlock) : lanes);
    lanes &= ~31u;
    ListTable<K> tab;
    tab.count = int(count);
    for (size_t i = 0; i < count; ++i) {
        ListEntry<K>& e = tab.e[i];
        for (int j = 0; j < K; ++j) e.in[j] = items[i].in[j];
        e.out = items[i].out;
        e.n = items[i].n;
        e.ntiles = items[i].n / T::kVec / lanes;
        e.trips = bulk_trips_per_burst(items[i].n, T::kVec, lanes, sh.grid, R);
        e.pad = 0;
    }
    const unsigned pace = sh.pace > 0 ? unsigned(sh.pace) : 0u;
    return launch_kernel(reduce_sum_bulk_list_kernel<T, K, R, kMaxBlock, SKEW>, dim3(sh.grid), dim3(lanes), stream, tab, pace);
}

template <typename T, int K>
hipError_t launch_reduce_bulk_list_k(const hfr_bucket* items, size_t count, const LaunchShape& sh, hipStream_t stream) {
    switch (sh.skew) {
        case 0: return launch_reduce_bulk_list_ks<T, K, 0>(items, count, sh, stream);
        case 3: return launch_reduce_bulk_list_ks<T, K, 3>(items, count, sh, stream);
        default: return hipErrorInvalidValue;  // the list kernels are built plain and with pattern 3
    }
}

template <typename T>
hipError_t launch_reduce_bulk_list(const hfr_bucket* items, size_t count, int K, const LaunchShape& sh,
                                   hipStream_t stream) {
    switch (K) {
        case 8: return launch_reduce_bulk_list_k<T, 8>(items, count, sh, stream);
        case 16: return launch_reduce_bulk_list_k<T, 16>(items, count, sh, stream);
        default: return hipErrorInvalidValue;
    }
}
#endif

#ifdef HFR_HEAVY_TU_MANY
template <typename T>
hipError_t launch_reduce_bulk_many(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                                   hipStream_t stream) {
    switch (K) {
        case 13: return launch_reduce_bulk_skew<T, 13, 0>(in, out, n, sh, stream);
        case 14: return launch_reduce_bulk_skew<T, 14, 0>(in, out, n, sh, stream);
        case 15: return launch_reduce_bulk_skew<T, 15, 0>(in, out, n, sh, stream);
        case 16: return launch_reduce_bulk_skew<T, 16, 0>(in, out, n, sh, stream);
        default: return hipErrorInvalidValue;
    }
}
#endif

#ifdef HFR_HEAVY_TU_SKEWED
template <typename T, int K>
hipError_t launch_reduce_bulk_skewed_k(const void* const* in, void* out, size_t n, const LaunchShape& sh,
                                       hipStream_t stream) {
    switch (sh.skew) {
        case 1: return launch_reduce_bulk_skew<T, K, 1>(in, out, n, sh, stream);
        case 2: return launch_reduce_bulk_skew<T, K, 2>(in, out, n, sh, stream);
        case 3: return launch_reduce_bulk_skew<T, K, 3>(in, out, n, sh, stream);
        default: return hipErrorInvalidValue;  // the plain kernel lives in the element type's main unit
    }
}

template <typename T>
hipError_t launch_reduce_bulk_skewed(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                                     hipStream_t stream) {
    switch (K) {
        case 8: return launch_reduce_bulk_skewed_k<T, 8>(in, out, n, sh, stream);
        case 9: return launch_reduce_bulk_skewed_k<T, 9>(in, out, n, sh, stream);
        default: return hipErrorInvalidValue;
    }
}
#endif

#ifdef HFR_HEAVY_TU_SKEWED3
template <typename T>
hipError_t launch_reduce_bulk_skewed3(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                                      hipStream_t stream) {
    if (sh.skew != 3) return hipErrorInvalidValue;
    switch (K) {
        case 5: return launch_reduce_bulk_skew<T, 5, 3, true>(in, out, n, sh, stream);
        case 6: return launch_reduce_bulk_skew<T, 6, 3, true>(in, out, n, sh, stream);
        case 7: return launch_reduce_bulk_skew<T, 7, 3, true>(in, out, n, sh, stream);
        case 10: return launch_reduce_bulk_skew<T, 10, 3, true>(in, out, n, sh, stream);
        case 11: return launch_reduce_bulk_skew<T, 11, 3, true>(in, out, n, sh, stream);
        case 12: return launch_reduce_bulk_skew<T, 12, 3, true>(in, out, n, sh, stream);
        case 13: return launch_reduce_bulk_skew<T, 13, 3, true>(in, out, n, sh, stream);
        case 14: return launch_reduce_bulk_skew<T, 14, 3, true>(in, out, n, sh, stream);
        case 15: return launch_reduce_bulk_skew<T, 15, 3, true>(in, out, n, sh, stream);
        case 16: return launch_reduce_bulk_skew<T, 16, 3, true>(in, out, n, sh, stream);
        default: return hipErrorInvalidValue;
    }
}
#endif

template <typename T, int K>
hipError_t launch_reduce_bulk_variant(const void* const* in, void* out, size_t n, const LaunchShape& sh,
                                      hipStream_t stream) {
    if (!sh.aligned16) return hipErrorInvalidValue;  // the host never picks the bulk shape then
    if constexpr (bulk_skew_available(K)) {
        if (sh.skew != 0) {
            if constexpr (bulk_skew_every_pattern(K))
                return launch_reduce_bulk_skewed<T>(in, K, out, n, sh, stream);
            else
                return launch_reduce_bulk_skewed3<T>(in, K, out, n, sh, stream);
        }
    }
    if constexpr (K > 12)
        return launch_reduce_bulk_many<T>(in, K, out, n, sh, stream);
    else
        return launch_reduce_bulk_skew<T, K, 0>(in, out, n, sh, stream);
}

template <typename T, int K, int U, int ELEM_ALIGN>
hipError_t launch_reduce_ku(const void* const* in, void* out, size_t n, const LaunchShape& sh,
                            hipStream_t stream) {
    if constexpr (U > max_unroll_for_k(K)) {
        return launch_reduce_ku<T, K, max_unroll_for_k(K), ELEM_ALIGN>(in, out, n, sh, stream);
    } else {
        if (sh.aligned16) return launch_reduce_variant<T, K, U, 16>(in, out, n, sh, stream);
        return launch_reduce_variant<T, K, U, ELEM_ALIGN>(in, out, n, sh, stream);
    }
}

template <typename T, int K, int ELEM_ALIGN>
hipError_t launch_reduce_k(const void* const* in, void* out, size_t n, const LaunchShape& sh,
                           hipStream_t stream) {
    if (sh.bulk) return launch_reduce_bulk_variant<T, K>(in, out, n, sh, stream);
    switch (sh.unroll) {
        case 4: return launch_reduce_ku<T, K, 4, ELEM_ALIGN>(in, out, n, sh, stream);
        case 2: return launch_reduce_ku<T, K, 2, ELEM_ALIGN>(in, out, n, sh, stream);
        default: return launch_reduce_ku<T, K, 1, ELEM_ALIGN>(in, out, n, sh, stream);
    }
}

template <typename T, int ELEM_ALIGN>
hipError_t launch_reduce_any_k(const void* const* in, int K, void* out, size_t n, const LaunchShape& sh,
                               hipStream_t stream) {
    switch (K) {
#define HFR_CASE_K(k) \
    case k: return launch_reduce_k<T, k, ELEM_ALIGN>(in, out, n, sh, stream);
        HFR_CASE_K(1) HFR_CASE_K(2) HFR_CASE_K(3) HFR_CASE_K(4)
        HFR_CASE_K(5) HFR_CASE_K(6) HFR_CASE_K(7) HFR_CASE_K(8)
        HFR_CASE_K(9) HFR_CASE_K(10) HFR_CASE_K(11) HFR_CASE_K(12)
        HFR_CASE_K(13) HFR_CASE_K(14) HFR_CASE_K(15) HFR_CASE_K(16)
#undef HFR_CASE_K
        default: return hipErrorInvalidValue;
    }
}

// Batched launch: `count` small buckets (count <= batch_capacity<K>()) in one grid.
// Tiles of 256 * U vectors; U as in the wide shape, halved while the launch
// would have fewer than eight tiles per compute unit.
template <typename T, int K, int U, int ELEM_ALIGN>
hipError_t launch_batched_ku(const hfr_bucket* buckets, size_t count, bool aligned16, size_t lds, hipStream_t stream) {
    constexpr size_t kVec = T::kVec;
    constexpr size_t kTile = size_t(kBlock) * U;
    static_assert(sizeof(BatchEntry<K>) == size_t(K + 3) * 8, "host and device agree on the table layout");
    static_assert(sizeof(BatchTable<K>) <= 3840, "the table fits the kernel-argument segment");
    if (count == 0 || count > size_t(batch_capacity<K>())) return hipErrorInvalidValue;
    BatchTable<K> tab;
    unsigned tiles = 0;
    for (size_t b = 0; b < count; ++b) {
        BatchEntry<K>& e = tab.e[b];
        for (int j = 0; j < K; ++j) e.in[j] = buckets[b].in[j];
        e.out = buckets[b].out;
        e.n = buckets[b].n;
        const size_t nvec = buckets[b].n / kVec;
        size_t nt = (nvec + kTile - 1) / kTile;
        if (nt == 0) nt = 1;  // tail only
        e.tile_begin = tiles;
        e.tile_count = unsigned(nt);
        tiles += unsigned(nt);
    }
    tab.count = int(count);
    auto launch = [&](size_t lds_bytes) -> hipError_t {
        if (aligned16)
            return launch_kernel_lds(reduce_sum_batched_kernel<T, K, U, kBlock, 16>, dim3(tiles), dim3(kBlock), lds_bytes, stream, tab);
        else
            return launch_kernel_lds(reduce_sum_batched_kernel<T, K, U, kBlock, ELEM_ALIGN>, dim3(tiles), dim3(kBlock), lds_bytes, stream, tab);
    };
    hipError_t e = launch(lds);
    if (e != hipSuccess && lds != 0) {
        // a runtime that refuses the reservation: the bound on resident workgroups is an optimisation only
        (void)hipGetLastError();
        e = launch(0);
    }
    return e;
}

template <typename T, int K, int ELEM_ALIGN>
hipError_t launch_batched_k(const hfr_bucket* buckets, size_t count, bool aligned16, hipStream_t stream) {
    int cus = 0;
    const hipError_t e = device_cu_count(&cus);
    if (e != hipSuccess) return e;
    size_t vecs = 0;
    for (size_t b = 0; b < count; ++b) vecs += buckets[b].n / T::kVec;
    int unroll = max_unroll_for_k(K);
    while (unroll > 1 && vecs / (size_t(kBlock) * unroll) < size_t(cus) * 8) unroll >>= 1;
    // the launch as a whole is one wide pass over `vecs` vectors per buffer: the same bound on
    // resident workgroups as a plain wide launch of that size
    const long knob = tuning().wide_wgs_per_cu.load();
    const int wgs = knob > 0 ? int(knob) : (knob < 0 ? 0 : default_wide_wgs_per_cu(K, vecs * 16));
    const size_t lds = lds_for_wgs_per_cu(wgs);
    if constexpr (max_unroll_for_k(K) >= 4) {
        if (unroll == 4) return launch_batched_ku<T, K, 4, ELEM_ALIGN>(buckets, count, aligned16, lds, stream);
    }
    if constexpr (max_unroll_for_k(K) >= 2) {
        if (unroll == 2) return launch_batched_ku<T, K, 2, ELEM_ALIGN>(buckets, count, aligned16, lds, stream);
    }
    return launch_batched_ku<T, K, 1, ELEM_ALIGN>(buckets, count, aligned16, lds, stream);
}

template <typename T, int ELEM_ALIGN>
hipError_t launch_batched_any_k(const hfr_bucket* buckets, size_t count, int K, bool aligned16,
                                hipStream_t stream) {
    switch (K) {
#define HFR_CASE_K(k) \
    case k: return launch_batched_k<T, k, ELEM_ALIGN>(buckets, count, aligned16, stream);
        HFR_CASE_K(1) HFR_CASE_K(2) HFR_CASE_K(3) HFR_CASE_K(4)
        HFR_CASE_K(5) HFR_CASE_K(6) HFR_CASE_K(7) HFR_CASE_K(8)
        HFR_CASE_K(9) HFR_CASE_K(10) HFR_CASE_K(11) HFR_CASE_K(12)
        HFR_CASE_K(13) HFR_CASE_K(14) HFR_CASE_K(15) HFR_CASE_K(16)
#undef HFR_CASE_K
        default: return hipErrorInvalidValue;
    }
}

template <typename T, int U, int ALIGN>
hipError_t launch_combine_variant(const void* a, const void* b, void* out, size_t n, float scale,
                                  unsigned grid, hipStream_t stream) {
    return launch_kernel(combine_avg_kernel<T, U, kBlock, ALIGN>, dim3(grid), dim3(kBlock), stream, a, b, out, n, scale);
}

template <typename T, int ALIGN>
hipError_t launch_combine_bulk_variant(const void* a, const void* b, void* out, size_t n, float scale,
                                       unsigned grid, hipStream_t stream) {
    constexpr int U = bulk_unroll_for_k(2);
    constexpr int R = bulk_result_vecs_for_k(2) / U;
    const unsigned trips = bulk_trips_per_burst(n, T::kVec, size_t(kBlock) * U, grid, R);
    return launch_kernel(combine_avg_bulk_kernel<T, U, R, kBlock, ALIGN>, dim3(grid), dim3(kBlock), stream, a, b, out, n, scale, trips);
}

template <typename T, int U, int ELEM_ALIGN>
hipError_t launch_combine_u(const void* a, const void* b, void* out, size_t n, float scale,
                            const LaunchShape& sh, hipStream_t stream) {
    if (sh.aligned16) return launch_combine_variant<T, U, 16>(a, b, out, n, scale, sh.grid, stream);
    return launch_combine_variant<T, U, ELEM_ALIGN>(a, b, out, n, scale, sh.grid, stream);
}

template <typename T, int ELEM_ALIGN>
hipError_t launch_combine_any(const void* a, const void* b, void* out, size_t n, float scale,
                              const LaunchShape& sh, hipStream_t stream) {
    if (sh.bulk) {
        if (!sh.aligned16) return hipErrorInvalidValue;  // the host never picks the bulk shape then
        return launch_combine_bulk_variant<T, 16>(a, b, out, n, scale, sh.grid, stream);
    }
    switch (sh.unroll) {
        case 4: return launch_combine_u<T, 4, ELEM_ALIGN>(a, b, out, n, scale, sh, stream);
        case 2: return launch_combine_u<T, 2, ELEM_ALIGN>(a, b, out, n, scale, sh, stream);
        default: return launch_combine_u<T, 1, ELEM_ALIGN>(a, b, out, n, scale, sh, stream);
    }
}

// Chunk table in device memory: grid x = tiles of a chunk of the hinted size
// (capped; longer chunks stride), grid y = chunks (capped; longer tables stride).
template <typename T, int K, int ELEM_ALIGN>
hipError_t launch_table_k(const void* table, size_t n_chunks, size_t chunk_elems_hint, hipStream_t stream) {
    constexpr int U = max_unroll_for_k(K);  // one variant per K: chunks shorter than a tile take the bounded path
    const size_t hint_vecs = chunk_elems_hint / T::kVec;
    const size_t tile = size_t(kBlock) * U;
    size_t gx = (hint_vecs + tile - 1) / tile;
    gx = gx < 1 ? 1 : (gx > 4096 ? 4096 : gx);
    const size_t gy = n_chunks < 65535 ? n_chunks : 65535;
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy)), block(kBlock);
    return launch_kernel(reduce_sum_table_kernel<T, K, U, kBlock, ELEM_ALIGN>, grid, block, stream, static_cast<const ChunkDesc*>(table), unsigned(n_chunks));
}

template <typename T, int ELEM_ALIGN>
hipError_t launch_table_any_k(const void* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                              hipStream_t stream) {
    switch (K) {
#define HFR_CASE_K(k) \
    case k: return launch_table_k<T, k, ELEM_ALIGN>(table, n_chunks, chunk_elems_hint, stream);
        HFR_CASE_K(1) HFR_CASE_K(2) HFR_CASE_K(3) HFR_CASE_K(4)
        HFR_CASE_K(5) HFR_CASE_K(6) HFR_CASE_K(7) HFR_CASE_K(8)
        HFR_CASE_K(9) HFR_CASE_K(10) HFR_CASE_K(11) HFR_CASE_K(12)
        HFR_CASE_K(13) HFR_CASE_K(14) HFR_CASE_K(15) HFR_CASE_K(16)
#undef HFR_CASE_K
        default: return hipErrorInvalidValue;
    }
}

}  // namespace hfr
