// The chunk-table reduction for callers that cannot allocate device memory:
// the table that hfr_reduce_chunk_table takes as a device buffer from its
// caller lives here in a file-scope device array instead. The host hands over
// the chunk list; small fill launches carry it in their kernel arguments and
// write it into the array; one launch of the table kernel then sums every
// chunk. No allocation, no host-to-device copy, nothing the host must keep
// alive after the call returns.
#include <stdint.h>
#include <stdio.h>

#include <mutex>

#include "hfr_internal.h"
#include "hfr_kernels.hip.h"

namespace hfr {

static_assert(sizeof(hfr_chunk) == sizeof(ChunkDesc), "host and device agree on the table entry");

// The staged chunk table of one GPU (each GPU that runs this code holds its own
// copy of the array until the process ends): HFR_NOALLOC_MAX_CHUNKS entries.
static __device__ __align__(256) unsigned char scratch[size_t(HFR_NOALLOC_MAX_CHUNKS) * sizeof(ChunkDesc)];

// Entries travel as packed 8-byte words, K + 2 per chunk (K input pointers,
// out, n), as many chunks per fill launch as the kernel-argument segment holds.
constexpr int kFillWords = 464;
struct FillWords {
    uint64_t w[kFillWords];
};

__global__ __launch_bounds__(512) void fill_chunk_table_kernel(ChunkDesc* table, FillWords words, unsigned first,
                                                               unsigned count, unsigned K) {
    const unsigned wpe = K + 2;  // words per entry
    const unsigned t = threadIdx.x;
    if (t >= count * wpe) return;
    const unsigned entry = t / wpe, field = t % wpe;
    uint64_t* dst = reinterpret_cast<uint64_t*>(table + first + entry);
    // fields 0..K-1 are in[0..K-1]; out and n sit behind the sixteen pointer slots
    dst[field < K ? field : 16 + (field - K)] = words.w[t];
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_setup_mutex;
ChunkDesc* g_table[kMaxDevices];  // device address of `scratch` on each device, once looked up
}  // namespace

// Looks up, once per device and with that device current, where this device's
// copy of the array lives. Host code never uses the array's name as an address:
// on the host it is only a handle for this query.
hfr_status noalloc_setup(ChunkDesc** table) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail_text(HFR_ERR_INVALID_ARG, "device index beyond the static table's bookkeeping");
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (g_table[dev] == nullptr) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        if (ptr == nullptr) return fail_text(HFR_ERR_HIP, "hipGetSymbolAddress(scratch) returned no address");
        g_table[dev] = static_cast<ChunkDesc*>(ptr);
    }
    if (table) *table = g_table[dev];
    return HFR_OK;
}

}  // namespace hfr

using namespace hfr;

extern "C" hfr_status hfr_reduce_chunks_noalloc(const hfr_chunk* chunks, size_t n_chunks, size_t chunk_elems_hint,
                                                int K, hfr_dtype dt, hipStream_t stream) {
    if (dtype_size(dt) == 0) return HFR_ERR_UNSUPPORTED_DTYPE;
    if (K < 1 || K > HFR_MAX_K) return HFR_ERR_INVALID_ARG;
    if (n_chunks == 0) return HFR_OK;
    if (chunks == nullptr || chunk_elems_hint == 0) return HFR_ERR_INVALID_ARG;
    if (n_chunks > size_t(HFR_NOALLOC_MAX_CHUNKS)) {
        char text[160];
        snprintf(text, sizeof text, "hfr_reduce_chunks_noalloc: %zu chunks exceed the static table's %d entries",
                 n_chunks, HFR_NOALLOC_MAX_CHUNKS);
        return fail_text(HFR_ERR_INVALID_ARG, text);
    }
    // the list is on the host here, so every chunk gets the checks hfr_reduce_sum makes
    for (size_t c = 0; c < n_chunks; ++c) {
        const hfr_status v = validate_reduce(chunks[c].in, K, chunks[c].out, chunks[c].n, dt);
        if (v != HFR_OK) return v;
    }
    ChunkDesc* table = nullptr;
    const hfr_status st = noalloc_setup(&table);
    if (st != HFR_OK) return st;

    const size_t wpe = size_t(K) + 2;
    const size_t per_launch = size_t(kFillWords) / wpe;
    FillWords words;
    for (size_t first = 0; first < n_chunks; first += per_launch) {
        const size_t count = n_chunks - first < per_launch ? n_chunks - first : per_launch;
        for (size_t c = 0; c < count; ++c) {
            const hfr_chunk& ch = chunks[first + c];
            uint64_t* w = words.w + c * wpe;
            for (int j = 0; j < K; ++j) w[j] = uint64_t(uintptr_t(ch.in[j]));
            w[K] = uint64_t(uintptr_t(ch.out));
            w[K + 1] = uint64_t(ch.n);  // every entry of this call is rewritten, n == 0 included
        }
        const hipError_t e = launch_kernel(fill_chunk_table_kernel, dim3(1), dim3(512), stream, table, words,
                                           unsigned(first), unsigned(count), unsigned(K));
        if (e != hipSuccess) return fail_hip(e, "chunk table fill launch");
    }
    const hipError_t e = dtype_ops(dt)->table(table, n_chunks, chunk_elems_hint, K, stream);
    if (e != hipSuccess) return fail_hip(e, "chunk table launch");
    return HFR_OK;
}
