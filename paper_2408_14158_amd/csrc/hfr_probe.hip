// Streaming probes (libhfr_probe.so): R read streams, W write streams, in the
// two launch shapes of the reduction kernels. Bytes only - vectors are XORed,
// nothing of the reduction arithmetic lives here. Used by the benchmark to
// measure what HBM delivers for a given read/write mix and access shape.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hfr_probe.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBlock = 256;

template <int N>
struct Ptrs {
    void* p[N > 0 ? N : 1];
};

__device__ __forceinline__ u32x4 ld(const void* p) { return __builtin_nontemporal_load(static_cast<const u32x4*>(p)); }
__device__ __forceinline__ void st(void* p, u32x4 v) { __builtin_nontemporal_store(v, static_cast<u32x4*>(p)); }

template <int R, int U>
__device__ __forceinline__ void load_tile(const Ptrs<R>& rd, size_t tile_byte, unsigned tid, unsigned block,
                                          u32x4 (&x)[U]) {
    if constexpr (R == 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = u32x4{0u, 0u, 0u, 0u};
    } else {
        u32x4 v[U][R];
#pragma unroll
        for (int j = 0; j < R; ++j)
#pragma unroll
            for (int u = 0; u < U; ++u)
                v[u][j] = ld(static_cast<const char*>(rd.p[j]) + tile_byte + (uint32_t(u) * block + tid) * 16u);
        __builtin_amdgcn_sched_barrier(0);  // every load of the trip goes out before the first use
#pragma unroll
        for (int u = 0; u < U; ++u) {
            x[u] = v[u][0];
#pragma unroll
            for (int j = 1; j < R; ++j) x[u] ^= v[u][j];
        }
    }
}

template <int W, int U>
__device__ __forceinline__ void store_tile(const Ptrs<W>& wr, size_t tile_byte, unsigned tid, unsigned block,
                                           const u32x4 (&x)[U]) {
#pragma unroll
    for (int j = 0; j < W; ++j)
#pragma unroll
        for (int u = 0; u < U; ++u)
            st(static_cast<char*>(wr.p[j]) + tile_byte + (uint32_t(u) * block + tid) * 16u, x[u]);
}

__device__ __forceinline__ bool is_marker(u32x4 v) {
    return v[0] == 0xDEADBEEFu && v[1] == 0xFEEDFACEu && v[2] == 0x0BADF00Du && v[3] == 0xCAFED00Du;
}

// Wide shape: workgroup b takes tiles b, b + grid, ...; stores follow their loads directly.
template <int R, int W, int U>
__global__ __launch_bounds__(kBlock) void probe_wide_kernel(Ptrs<R> rd, Ptrs<W> wr, void* sink, size_t ntiles) {
    const unsigned tid = threadIdx.x;
    constexpr size_t kTileBytes = size_t(kBlock) * U * 16;
    u32x4 seen = {0u, 0u, 0u, 0u};
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        u32x4 x[U];
        load_tile<R, U>(rd, tile * kTileBytes, tid, kBlock, x);
        if constexpr (W > 0) {
            store_tile<W, U>(wr, tile * kTileBytes, tid, kBlock, x);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) seen ^= x[u];
        }
    }
    if constexpr (W == 0) {
        if (is_marker(seen)) st(sink, seen);
    }
}

// Bulk shape: one workgroup per compute unit; tiles b, b + G, ... in lock step
// with the other workgroups; P trips' results parked in registers and stored in
// one burst (P * U = 32 vectors per lane, as the library's bulk kernels). As in
// the library, the workgroup size is a run-time value (a tile is blockDim.x * U
// vectors) and a workgroup may pause for pace * 64 clocks after each trip: the
// two knobs that set how many loads a compute unit keeps in flight.
constexpr int kMaxBulkBlock = 384;
template <int R, int W, int U>
__global__ __launch_bounds__(kMaxBulkBlock) void probe_bulk_kernel(Ptrs<R> rd, Ptrs<W> wr, void* sink, size_t ntiles,
                                                                   unsigned trips, unsigned pace) {
    constexpr int P = 32 / U;
    const unsigned tid = threadIdx.x;
    const unsigned block = blockDim.x;
    const size_t G = gridDim.x;
    const size_t kTileBytes = size_t(block) * U * 16;
    trips = trips < 1u ? 1u : (trips > unsigned(P) ? unsigned(P) : trips);  // the loop below must advance
    u32x4 seen = {0u, 0u, 0u, 0u};
    for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
        u32x4 res[P][U];
#pragma unroll
        for (int r = 0; r < P; ++r) {
            const size_t tile = t0 + G * r;
            if (unsigned(r) < trips && tile < ntiles) {
                load_tile<R, U>(rd, tile * kTileBytes, tid, block, res[r]);
                for (unsigned i = 0; i < pace; ++i) __builtin_amdgcn_s_sleep(1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < P; ++r) {
            const size_t tile = t0 + G * r;
            if (unsigned(r) < trips && tile < ntiles) {
                if constexpr (W > 0) {
                    store_tile<W, U>(wr, tile * kTileBytes, tid, block, res[r]);
                } else {
#pragma unroll
                    for (int u = 0; u < U; ++u) seen ^= res[r][u];
                }
            }
        }
    }
    if constexpr (W == 0) {
        if (is_marker(seen)) st(sink, seen);
    }
}

// vectors per lane and trip: as the library chooses them for a K-input sum
constexpr int unroll_for(int streams) { return streams <= 1 ? 8 : (streams == 2 ? 4 : (streams <= 4 ? 2 : 1)); }

template <int R, int W>
hipError_t launch(const void* const* rd, void* const* wr, void* sink, size_t nbytes, int shape, unsigned lanes,
                  unsigned pace, hipStream_t stream) {
    constexpr int U = unroll_for(R > W ? R : W);
    Ptrs<R> r;
    Ptrs<W> w;
    for (int j = 0; j < R; ++j) r.p[j] = const_cast<void*>(rd[j]);
    for (int j = 0; j < W; ++j) w.p[j] = wr[j];
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (cus < 1) cus = 1;
    if (shape == HFR_PROBE_BULK) {
        const size_t ntiles = nbytes / (size_t(lanes) * U * 16);  // whole tiles only
        const size_t grid = ntiles < size_t(cus) ? (ntiles ? ntiles : 1) : size_t(cus);
        constexpr size_t P = 32 / U;
        size_t per_wg = (ntiles + grid - 1) / grid;
        if (per_wg == 0) per_wg = 1;
        const size_t bursts = (per_wg + P - 1) / P;
        unsigned trips = unsigned((per_wg + bursts - 1) / bursts);  // split evenly over the bursts
        void* args[] = {&r, &w, &sink, const_cast<size_t*>(&ntiles), &trips, &pace};
        return hipLaunchKernel(reinterpret_cast<const void*>(&probe_bulk_kernel<R, W, U>), dim3(unsigned(grid)),
                               dim3(lanes), args, 0, stream);
    }
    const size_t ntiles = nbytes / (size_t(kBlock) * U * 16);
    void* args_wide[] = {&r, &w, &sink, const_cast<size_t*>(&ntiles)};
    const size_t cap = size_t(cus) * 16;
    const size_t grid = ntiles < cap ? (ntiles ? ntiles : 1) : cap;
    return hipLaunchKernel(reinterpret_cast<const void*>(&probe_wide_kernel<R, W, U>), dim3(unsigned(grid)),
                           dim3(kBlock), args_wide, 0, stream);
}

template <int W>
hipError_t launch_r(const void* const* rd, int R, void* const* wr, void* sink, size_t nbytes, int shape,
                    unsigned lanes, unsigned pace, hipStream_t stream) {
    switch (R) {
#define HFR_CASE(r) \
    case r: return launch<r, W>(rd, wr, sink, nbytes, shape, lanes, pace, stream);
        HFR_CASE(0) HFR_CASE(1) HFR_CASE(2) HFR_CASE(3) HFR_CASE(4) HFR_CASE(5) HFR_CASE(6) HFR_CASE(7) HFR_CASE(8)
        HFR_CASE(9) HFR_CASE(10) HFR_CASE(11) HFR_CASE(12) HFR_CASE(13) HFR_CASE(14) HFR_CASE(15) HFR_CASE(16)
#undef HFR_CASE
        default: return hipErrorInvalidValue;
    }
}

template <int R>
hipError_t launch_w(const void* const* rd, void* const* wr, int W, void* sink, size_t nbytes, int shape,
                    unsigned lanes, unsigned pace, hipStream_t stream) {
    switch (W) {
#define HFR_CASE(w) \
    case w: return launch<R, w>(rd, wr, sink, nbytes, shape, lanes, pace, stream);
        HFR_CASE(2) HFR_CASE(3) HFR_CASE(4) HFR_CASE(5) HFR_CASE(6) HFR_CASE(7) HFR_CASE(8)
        HFR_CASE(9) HFR_CASE(10) HFR_CASE(11) HFR_CASE(12) HFR_CASE(13) HFR_CASE(14) HFR_CASE(15) HFR_CASE(16)
#undef HFR_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

static int probe_stream(const void* const* rd, int n_read, void* const* wr, int n_write, void* sink, size_t nbytes,
                        int shape, unsigned lanes, unsigned pace, hipStream_t stream) {
    if (n_read < 0 || n_read > HFR_PROBE_MAX_STREAMS || n_write < 0 || n_write > HFR_PROBE_MAX_STREAMS) return 1;
    if (n_read + n_write == 0 || (n_read > 1 && n_write > 1)) return 1;
    if (nbytes == 0 || nbytes % (size_t(kBlock) * 8 * 16) != 0) return 1;
    if (shape != HFR_PROBE_WIDE && shape != HFR_PROBE_BULK) return 1;
    if (lanes < 64 || lanes > unsigned(kMaxBulkBlock) || lanes % 32 != 0 || pace > 64) return 1;
    if ((n_read > 0 && rd == nullptr) || (n_write > 0 && wr == nullptr)) return 1;
    if (n_write == 0 && sink == nullptr) return 1;
    for (int j = 0; j < n_read; ++j)
        if (rd[j] == nullptr || (reinterpret_cast<uintptr_t>(rd[j]) & 15) != 0) return 1;
    for (int j = 0; j < n_write; ++j)
        if (wr[j] == nullptr || (reinterpret_cast<uintptr_t>(wr[j]) & 15) != 0) return 1;
    hipError_t e;
    if (n_write == 0) e = launch_r<0>(rd, n_read, wr, sink, nbytes, shape, lanes, pace, stream);
    else if (n_write == 1) e = launch_r<1>(rd, n_read, wr, sink, nbytes, shape, lanes, pace, stream);
    else if (n_read == 0) e = launch_w<0>(rd, wr, n_write, sink, nbytes, shape, lanes, pace, stream);
    else e = launch_w<1>(rd, wr, n_write, sink, nbytes, shape, lanes, pace, stream);
    return e == hipSuccess ? 0 : 5;
}

extern "C" int hfr_probe_stream(const void* const* rd, int n_read, void* const* wr, int n_write, void* sink,
                                size_t nbytes, hfr_probe_shape shape, hipStream_t stream) {
    return probe_stream(rd, n_read, wr, n_write, sink, nbytes, int(shape), unsigned(kBlock), 0u, stream);
}

extern "C" int hfr_probe_stream_paced(const void* const* rd, int n_read, void* const* wr, int n_write, void* sink,
                                      size_t nbytes, int lanes, int pace, hipStream_t stream) {
    if (lanes < 0 || pace < 0) return 1;
    return probe_stream(rd, n_read, wr, n_write, sink, nbytes, int(HFR_PROBE_BULK), unsigned(lanes), unsigned(pace),
                        stream);
}
