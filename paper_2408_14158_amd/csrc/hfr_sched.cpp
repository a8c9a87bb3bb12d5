// Chunk scheduler of libhfr: Algorithm 1's outer loop (cut by Chunk_Size, reduce
// chunk after chunk) over a list of gradient buckets, pipelined over a ring of
// HIP streams. Worker streams fork from the caller's stream with one event and
// join back with one event each, so the host never blocks and the caller sees
// plain stream order.
#include <stdint.h>

#include <mutex>
#include <vector>

#include "hfr_internal.h"

namespace hfr {

struct StreamPool {
    int device = -1;
    std::mutex mutex;  // one fork/join sequence at a time per device
    std::vector<hipStream_t> streams;
    std::vector<hipEvent_t> joins;
    hipEvent_t fork = nullptr;
};

static std::mutex g_pools_mutex;
static std::vector<StreamPool*> g_pools;

hfr_status pool_acquire(int n_streams, StreamPool** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    StreamPool* pool = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_pools_mutex);
        for (StreamPool* p : g_pools)
            if (p->device == dev) pool = p;
        if (pool == nullptr) {
            pool = new StreamPool();
            pool->device = dev;
            g_pools.push_back(pool);
        }
    }
    // The pool stays locked from here until the caller's pool_unlock(): the streams
    // this call made sure of cannot be destroyed (hfr_shutdown from another thread)
    // between now and their use.
    pool->mutex.lock();
    if (pool->fork == nullptr) {
        e = hipEventCreateWithFlags(&pool->fork, hipEventDisableTiming);
        if (e != hipSuccess) {
            pool->mutex.unlock();
            return fail_hip(e, "hipEventCreate");
        }
    }
    while (int(pool->streams.size()) < n_streams) {
        hipStream_t s = nullptr;
        hipEvent_t ev = nullptr;
        // default priority; non-blocking so the null stream does not serialise the ring
        e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
        if (e == hipSuccess) {
            e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
            if (e != hipSuccess) (void)hipStreamDestroy(s);
        }
        if (e != hipSuccess) {
            pool->mutex.unlock();
            return fail_hip(e, "worker stream set-up");
        }
        pool->streams.push_back(s);
        pool->joins.push_back(ev);
    }
    *out = pool;
    return HFR_OK;
}

hipStream_t pool_stream(StreamPool* pool, int w) { return pool->streams[size_t(w)]; }
hipEvent_t pool_fork_event(StreamPool* pool) { return pool->fork; }
hipEvent_t pool_join_event(StreamPool* pool, int w) { return pool->joins[size_t(w)]; }
void pool_unlock(StreamPool* pool) { pool->mutex.unlock(); }

hfr_status pool_destroy_all() {
    std::lock_guard<std::mutex> lock(g_pools_mutex);
    hfr_status st = HFR_OK;
    int prev = 0;
    const bool have_prev = hipGetDevice(&prev) == hipSuccess;
    for (StreamPool* p : g_pools) {
        std::lock_guard<std::mutex> plock(p->mutex);
        if (hipSetDevice(p->device) != hipSuccess) continue;
        for (hipStream_t s : p->streams) {
            const hipError_t e = hipStreamDestroy(s);
            if (e != hipSuccess) st = fail_hip(e, "hipStreamDestroy");
        }
        for (hipEvent_t ev : p->joins) (void)hipEventDestroy(ev);
        if (p->fork) (void)hipEventDestroy(p->fork);
        p->streams.clear();
        p->joins.clear();
        p->fork = nullptr;
    }
    // pool objects stay allocated: another thread may still hold a pointer
    if (have_prev) (void)hipSetDevice(prev);
    return st;
}

}  // namespace hfr

using namespace hfr;

extern "C" {

// A chunk whose whole traffic (K reads and one write) is at most 16 MiB runs
// for a few microseconds: short enough that it does not disturb a bulk launch
// it overlaps with, and launch-latency bound on its own.
static bool chunk_is_tiny(int K, size_t len, size_t es) {
    return (size_t(K) + 1) * len * es <= (size_t(16) << 20);
}
// Up to about 96 MiB of traffic (some 15 microseconds) a chunk gains from
// running beside its neighbours on other streams: their launch, ramp-up and
// tail overlap (measured: 5 to 10 % for K = 8 at 4 to 8 MiB per buffer).
// Longer chunks fill the GPU on their own and side by side only get in each
// other's way (measured: -6 to -10 % at 12 to 24 MiB per buffer).
static bool chunk_gains_from_ring(int K, size_t len, size_t es) {
    return (size_t(K) + 1) * len * es <= (size_t(96) << 20);
}

hfr_status hfr_reduce_buckets(const hfr_bucket* buckets, size_t n_buckets, int K, hfr_dtype dt,
                              size_t chunk_elems, int n_streams, hipStream_t stream) {
    const size_t es = dtype_size(dt);
    if (es == 0) return HFR_ERR_UNSUPPORTED_DTYPE;
    if (K < 1 || K > HFR_MAX_K) return HFR_ERR_INVALID_ARG;
    if (chunk_elems == 0) return HFR_ERR_INVALID_ARG;
    if (n_streams < 1 || n_streams > HFR_MAX_STREAMS) return HFR_ERR_INVALID_ARG;
    if (n_buckets == 0) return HFR_OK;
    if (buckets == nullptr) return HFR_ERR_INVALID_ARG;

    // validate everything before the first enqueue, and sort the chunks into
    // "bulk" (big enough to occupy the whole GPU alone), tiny ones (a few
    // microseconds of work) and the rest
    size_t ringable_chunks = 0, tiny_chunks = 0, all_chunks = 0;
    bool has_bulk = false;
    for (size_t b = 0; b < n_buckets; ++b) {
        const hfr_status v = validate_reduce(buckets[b].in, K, buckets[b].out, buckets[b].n, dt);
        if (v != HFR_OK) return v;
        for (size_t off = 0; off < buckets[b].n; off += chunk_elems) {
            const size_t len = buckets[b].n - off < chunk_elems ? buckets[b].n - off : chunk_elems;
            bool bulk = false;
            if (n_streams > 1) {
                const hfr_status st = reduce_is_bulk(K, len, dt, &bulk);
                if (st != HFR_OK) return st;
            }
            ++all_chunks;
            if (bulk) has_bulk = true;
            else {
                if (chunk_gains_from_ring(K, len, es)) ++ringable_chunks;
                if (chunk_is_tiny(K, len, es)) ++tiny_chunks;
            }
        }
    }
    if (all_chunks == 0) return HFR_OK;

    // Small chunks go round the ring so that their launch and ramp-up gaps
    // overlap. A bulk chunk owns every compute unit while it runs and depends
    // on its workgroups moving in lock step: another launch beside it (bulk or
    // not) slows both down, and a hop to another stream costs more than the gap
    // it could hide, so bulk chunks stay in order on the caller's stream, and
    // in a call that has bulk chunks only tiny chunks may run beside them.
    // Mid-size chunks that fill the GPU on their own stay on the caller's
    // stream as well. The ring is forked only when it has work.
    const size_t ring_chunks = has_bulk ? tiny_chunks : ringable_chunks;
    const bool ring = n_streams > 1 && ring_chunks > 1;
    StreamPool* pool = nullptr;
    int used = 1;
    if (ring) {
        used = ring_chunks < size_t(n_streams) ? int(ring_chunks) : n_streams;
        const hfr_status st = pool_acquire(used, &pool);  // locked on success
        if (st != HFR_OK) return st;
        hipError_t e = hipEventRecord(pool_fork_event(pool), stream);
        for (int w = 0; e == hipSuccess && w < used; ++w)
            e = hipStreamWaitEvent(pool_stream(pool, w), pool_fork_event(pool), 0);
        if (e != hipSuccess) {
            pool_unlock(pool);
            return fail_hip(e, "fork");
        }
    }

    hfr_status result = HFR_OK;
    size_t c = 0;
    const void* chunk_in[HFR_MAX_K];
    for (size_t b = 0; b < n_buckets && result == HFR_OK; ++b) {
        const hfr_bucket& bk = buckets[b];
        for (size_t off = 0; off < bk.n && result == HFR_OK; off += chunk_elems) {
            const size_t len = bk.n - off < chunk_elems ? bk.n - off : chunk_elems;
            for (int j = 0; j < K; ++j) chunk_in[j] = static_cast<const char*>(bk.in[j]) + off * es;
            void* chunk_out = static_cast<char*>(bk.out) + off * es;
            hipStream_t s = stream;
            if (ring) {
                bool bulk = false;
                result = reduce_is_bulk(K, len, dt, &bulk);
                if (result != HFR_OK) break;
                const bool to_ring = !bulk && (has_bulk ? chunk_is_tiny(K, len, es) : chunk_gains_from_ring(K, len, es));
                if (to_ring) s = pool_stream(pool, int(c++ % size_t(used)));
            }
            result = enqueue_reduce(chunk_in, K, chunk_out, len, dt, s);
        }
    }

    if (ring) {
        // join even after a failed launch so the caller's stream stays ordered
        for (int w = 0; w < used; ++w) {
            hipError_t e = hipEventRecord(pool_join_event(pool, w), pool_stream(pool, w));
            if (e == hipSuccess) e = hipStreamWaitEvent(stream, pool_join_event(pool, w), 0);
            if (e != hipSuccess && result == HFR_OK) result = fail_hip(e, "join");
        }
        pool_unlock(pool);
    }
    return result;
}

hfr_status hfr_reduce_buckets_batched(const hfr_bucket* buckets, size_t n_buckets, int K, hfr_dtype dt,
                                      hipStream_t stream) {
    const size_t es = dtype_size(dt);
    if (es == 0) return HFR_ERR_UNSUPPORTED_DTYPE;
    if (K < 1 || K > HFR_MAX_K) return HFR_ERR_INVALID_ARG;
    if (n_buckets == 0) return HFR_OK;
    if (buckets == nullptr) return HFR_ERR_INVALID_ARG;
    for (size_t b = 0; b < n_buckets; ++b) {
        const hfr_status v = validate_reduce(buckets[b].in, K, buckets[b].out, buckets[b].n, dt);
        if (v != HFR_OK) return v;
    }

    const size_t cap = batch_capacity(K);
    size_t first = 0, pending = 0;  // buckets [first, first + pending) wait for one batched launch
    bool pending_aligned = true;
    auto flush = [&]() -> hfr_status {
        if (pending == 0) return HFR_OK;
        const hipError_t e = dtype_ops(dt)->batched(buckets + first, pending, K, pending_aligned, stream);
        pending = 0;
        pending_aligned = true;
        return e == hipSuccess ? HFR_OK : fail_hip(e, "batched launch");
    };
    for (size_t b = 0; b < n_buckets; ++b) {
        const hfr_bucket& bk = buckets[b];
        const bool small = bk.n * es <= kBatchMaxBytes;
        if (bk.n == 0 || !small) {
            // empty: nothing to do; big: worth a launch of its own (order on the stream is kept)
            const hfr_status st = flush();
            if (st != HFR_OK) return st;
            if (bk.n != 0) {
                const hfr_status r = enqueue_reduce(bk.in, K, bk.out, bk.n, dt, stream);
                if (r != HFR_OK) return r;
            }
            continue;
        }
        if (pending == 0) first = b;
        uintptr_t bits = uintptr_t(bk.out);
        for (int j = 0; j < K; ++j) bits |= uintptr_t(bk.in[j]);
        pending_aligned = pending_aligned && (bits & 15) == 0;
        if (++pending == cap) {
            const hfr_status st = flush();
            if (st != HFR_OK) return st;
        }
    }
    return flush();
}

hfr_status hfr_init(void) {
    StreamPool* pool = nullptr;
    const hfr_status st = pool_acquire(4, &pool);
    if (st == HFR_OK) pool_unlock(pool);
    return st;
}

hfr_status hfr_shutdown(void) {
    placement_clear();
    return pool_destroy_all();
}

}  // extern "C"
