// Broadcast kernel variants and their launcher (type-agnostic byte movers).
#include "hfr_internal.h"
#include "hfr_kernels.hip.h"

namespace hfr {

template <int K, int U>
static hipError_t launch_broadcast_ku(const void* src, void* const* dst, size_t nbytes, bool aligned16,
                                      unsigned grid, hipStream_t stream) {
    DstPack<K> pack;
    for (int j = 0; j < K; ++j) pack.p[j] = dst[j];
    if (aligned16)
        return launch_kernel(broadcast_kernel<K, U, kBlock, 16>, dim3(grid), dim3(kBlock), stream, src, pack, nbytes);
    else
        return launch_kernel(broadcast_kernel<K, U, kBlock, 1>, dim3(grid), dim3(kBlock), stream, src, pack, nbytes);
}

// From three destinations and 20 MiB per buffer (16-byte aligned) the bulk shape wins: the
// workgroups park 32 tiles in registers and write one destination after the other.
constexpr int kBroadcastParked = 32;
constexpr size_t kBroadcastBulkMinBytes = size_t(20) << 20;

template <int K>
static hipError_t launch_broadcast_bulk(const void* src, void* const* dst, size_t nbytes, int cus,
                                        hipStream_t stream) {
    DstPack<K> pack;
    for (int j = 0; j < K; ++j) pack.p[j] = dst[j];
    const size_t ntiles = nbytes / 16 / kBlock;
    const long knob = tuning().bulk_grid.load();
    const size_t want = knob > 0 ? size_t(knob) : size_t(cus);
    const size_t grid = ntiles < want ? (ntiles > 0 ? ntiles : 1) : want;
    size_t per_wg = (ntiles + grid - 1) / grid;
    if (per_wg == 0) per_wg = 1;
    const size_t bursts = (per_wg + kBroadcastParked - 1) / kBroadcastParked;
    const unsigned trips = unsigned((per_wg + bursts - 1) / bursts);  // split evenly over the bursts
    return launch_kernel(broadcast_bulk_kernel<K, kBroadcastParked, kBlock>, dim3(unsigned(grid)), dim3(kBlock), stream, src, pack, nbytes, trips);
}

template <int K>
static hipError_t launch_broadcast_k(const void* src, void* const* dst, size_t nbytes, bool aligned16,
                                     int cus, hipStream_t stream) {
    if constexpr (K >= 3) {
        const long forced = tuning().bulk_min_bytes.load();  // the knob of the sums applies here too
        const bool bulk = forced > 0 ? nbytes >= size_t(forced) : (forced == 0 && nbytes >= kBroadcastBulkMinBytes);
        if (aligned16 && bulk) return launch_broadcast_bulk<K>(src, dst, nbytes, cus, stream);
    }
    // one load stream only: four vectors per lane in flight unless the input is too small to fill the chip
    const size_t nvec = nbytes / 16;
    int unroll = 4;
    while (unroll > 1 && nvec / (size_t(kBlock) * unroll) < size_t(cus) * 4) unroll >>= 1;
    const size_t tile = size_t(kBlock) * unroll;
    size_t ntiles = (nvec + tile - 1) / tile;
    if (ntiles == 0) ntiles = 1;
    const size_t cap = size_t(cus) * 16;
    const unsigned grid = unsigned(ntiles < cap ? ntiles : cap);
    switch (unroll) {
        case 4: return launch_broadcast_ku<K, 4>(src, dst, nbytes, aligned16, grid, stream);
        case 2: return launch_broadcast_ku<K, 2>(src, dst, nbytes, aligned16, grid, stream);
        default: return launch_broadcast_ku<K, 1>(src, dst, nbytes, aligned16, grid, stream);
    }
}

hipError_t launch_broadcast(const void* src, void* const* dst, int K, size_t nbytes, bool aligned16,
                            hipStream_t stream) {
    int cus = 0;
    const hipError_t e = device_cu_count(&cus);
    if (e != hipSuccess) return e;
    switch (K) {
#define HFR_CASE_K(k) \
    case k: return launch_broadcast_k<k>(src, dst, nbytes, aligned16, cus, stream);
        HFR_CASE_K(1) HFR_CASE_K(2) HFR_CASE_K(3) HFR_CASE_K(4)
        HFR_CASE_K(5) HFR_CASE_K(6) HFR_CASE_K(7) HFR_CASE_K(8)
        HFR_CASE_K(9) HFR_CASE_K(10) HFR_CASE_K(11) HFR_CASE_K(12)
        HFR_CASE_K(13) HFR_CASE_K(14) HFR_CASE_K(15) HFR_CASE_K(16)
#undef HFR_CASE_K
        default: return hipErrorInvalidValue;
    }
}

}  // namespace hfr
