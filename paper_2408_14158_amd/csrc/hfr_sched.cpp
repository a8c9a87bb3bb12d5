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
// Chunks of up to 8 MiB per buffer are folded into batched launches (one grid
// over many chunks, chunk table in the kernel arguments): a launch per chunk
// costs the host about 3 microseconds, more than such a chunk runs for.
static bool chunk_is_batchable(size_t len, size_t es) { return len * es <= kBatchMaxBytes; }
// Mid-size chunks that lie apart (adjacent ones have been merged before this is asked) may run
// together as bulk launches over a list of chunks where such kernels exist (8 and 16 inputs,
// 16-byte aligned buffers): against a launch per chunk the chip does not drain between chunks.
// Measured on 64 chunks 4 KiB apart, plain kernels, bf16 / fp32, list launches against the schedule
// without them: K = 8: 12 MiB per buffer +6 / +4 %, 16 MiB +3 / +2 %, 20 MiB +5 / +4 %, 24 MiB
// +7 / +2 %, 32 MiB +2 / 0 %; K = 16: 6 MiB +4 / +10 %, 8 MiB +6 / +7 %, 12 MiB +8 / +11 %, 16 MiB
// +3 / +5 %, 20 MiB +2 / +4 %. Below that the batched launch of the wide shape wins (K = 8 at 8 MiB:
// -11 / -7 %, at 4 MiB -27 / -24 %), above it a launch per chunk is as good. This is the size rule;
// hfr_reduce_buckets adds the placement rule (the plain kernel must be the recorded best).
static bool chunk_is_listable(int K, size_t len, size_t es, bool aligned16, long knob) {
    if (knob < 0 || !aligned16 || !list_available(K)) return false;
    if (knob > 0) return true;
    const size_t mib = size_t(1) << 20, bytes = len * es;
    return K > 12 ? bytes >= 5 * mib && bytes < 24 * mib : bytes >= 10 * mib && bytes < 32 * mib;
}

namespace {
// Small chunks waiting for one batched launch. The pointer rows live in one
// array sized for a full table, so the descriptors' `in` pointers stay valid.
struct ChunkBatch {
    std::vector<const void*> rows;
    std::vector<hfr_bucket> items;
    size_t count = 0;
    bool aligned16 = true;
    void reset(size_t cap, int K) {
        if (rows.size() < cap * size_t(K)) rows.resize(cap * size_t(K));
        if (items.size() < cap) items.resize(cap);
        count = 0;
        aligned16 = true;
    }
    void add(const void* const* in, int K, void* out, size_t n) {
        const void** row = rows.data() + count * size_t(K);
        uintptr_t bits = uintptr_t(out);
        for (int j = 0; j < K; ++j) {
            row[j] = in[j];
            bits |= uintptr_t(in[j]);
        }
        items[count].in = row;
        items[count].out = out;
        items[count].n = n;
        aligned16 = aligned16 && (bits & 15) == 0;
        ++count;
    }
};
// A run of chunks that follow each other in memory - every input and the output
// of the next chunk start where the previous chunk's end - and are launched as
// one longer elementwise sum.
struct ChunkRun {
    const void* in[HFR_MAX_K];
    void* out = nullptr;
    size_t n = 0;  // elements so far; 0: no run is open
    void start(const void* const* cin, int K, void* cout, size_t len) {
        for (int j = 0; j < K; ++j) in[j] = cin[j];
        out = cout;
        n = len;
    }
    // The next chunk continues the run, and the longer run still has no input that overlaps the
    // output partially.
    bool continued_by(const void* const* cin, int K, const void* cout, size_t len, size_t es) const {
        if (n == 0) return false;
        const size_t bytes = n * es, total = (n + len) * es;
        if (static_cast<const char*>(out) + bytes != cout) return false;
        for (int j = 0; j < K; ++j)
            if (static_cast<const char*>(in[j]) + bytes != cin[j]) return false;
        for (int j = 0; j < K; ++j) {
            const uintptr_t a = uintptr_t(in[j]), o = uintptr_t(out);
            if (a != o && (a > o ? a - o : o - a) < total) return false;
        }
        return true;
    }
};
}  // namespace

hfr_status hfr_reduce_buckets(const hfr_bucket* buckets, size_t n_buckets, int K, hfr_dtype dt,
                              size_t chunk_elems, int n_streams, hipStream_t stream) {
    const size_t es = dtype_size(dt);
    if (es == 0) return HFR_ERR_UNSUPPORTED_DTYPE;
    if (K < 1 || K > HFR_MAX_K) return HFR_ERR_INVALID_ARG;
    if (chunk_elems == 0) return HFR_ERR_INVALID_ARG;
    if (n_streams < 1 || n_streams > HFR_MAX_STREAMS) return HFR_ERR_INVALID_ARG;
    if (n_buckets == 0) return HFR_OK;
    if (buckets == nullptr) return HFR_ERR_INVALID_ARG;

    // Validate everything before the first enqueue.
    size_t all_chunks = 0;
    for (size_t b = 0; b < n_buckets; ++b) {
        const hfr_status v = validate_reduce(buckets[b].in, K, buckets[b].out, buckets[b].n, dt);
        if (v != HFR_OK) return v;
        all_chunks += (buckets[b].n + chunk_elems - 1) / chunk_elems;
    }
    if (all_chunks == 0) return HFR_OK;
    const long fold_knob = tuning().bucket_fold.load();
    const bool fold = fold_knob >= 0;

    // Chunks that follow each other in memory - every input and the output of the next chunk start
    // where the previous chunk's end, as the chunks of one bucket and buckets cut from one flat
    // buffer do - are one longer elementwise sum and are handled as ONE chunk of the summed length
    // (a "run"): the bits are the same element by element, small chunks need no table entry each,
    // and for large ones every launch boundary costs the start-up of a launch on pages the chip has
    // not translated yet (measured on 3.3 GiB buffers, K = 8 bf16: launches of 50 MiB per buffer
    // 6.49 TB/s, of 128 MiB 6.68; on one 50 MiB chunk over and over, whose pages stay translated,
    // the two differ by 0.5 %). enqueue_reduce cuts a long run into its segments. `walk` hands every
    // run of the list to `emit`, in list order.
    const void* chunk_in[HFR_MAX_K];
    auto walk = [&](auto&& emit) -> hfr_status {
        ChunkRun run;
        for (size_t b = 0; b < n_buckets; ++b) {
            const hfr_bucket& bk = buckets[b];
            for (size_t off = 0; off < bk.n; off += chunk_elems) {
                const size_t len = bk.n - off < chunk_elems ? bk.n - off : chunk_elems;
                for (int j = 0; j < K; ++j) chunk_in[j] = static_cast<const char*>(bk.in[j]) + off * es;
                void* chunk_out = static_cast<char*>(bk.out) + off * es;
                if (fold && run.continued_by(chunk_in, K, chunk_out, len, es)) {
                    run.n += len;
                    continue;
                }
                if (run.n != 0) {
                    const hfr_status st = emit(run);
                    if (st != HFR_OK) return st;
                }
                run.start(chunk_in, K, chunk_out, len);
            }
        }
        return run.n != 0 ? emit(run) : HFR_OK;
    };

    // Where each run goes. A run is "bulk" (big enough to occupy the whole GPU
    // alone: in order on the caller's stream), or small enough to be folded with
    // others into a batched launch, or it keeps a launch of its own, on the
    // worker ring if it gains from running beside its neighbours and on the
    // caller's stream otherwise.
    size_t memo_len = 0;  // runs of a call mostly share one length
    bool memo_bulk = false;
    hfr_status memo_status = HFR_OK;
    auto is_bulk = [&](size_t len) {
        if (len != memo_len) {
            memo_len = len;
            memo_status = reduce_is_bulk(K, len, dt, &memo_bulk);
        }
        return memo_bulk;
    };
    const long list_knob = fold ? tuning().bucket_list.load() : -1;
    auto run_aligned16 = [&](const ChunkRun& run) {
        uintptr_t bits = uintptr_t(run.out);
        for (int j = 0; j < K; ++j) bits |= uintptr_t(run.in[j]);
        return (bits & 15) == 0;
    };
    // The list kernels are built plain and with skew pattern 3. By default a chunk joins a list only
    // where the placement table has recorded one of the two as the best variant for its buffers, and
    // the list launch runs that variant (on a placement that wants a skewed variant the plain list
    // kernel loses to a launch per chunk with that variant: 25 MiB buckets in buffers about 1 GiB
    // apart 6.5 TB/s against 6.2, and 5.7 with plain launches per chunk). Returns the variant, or
    // -1 for a chunk that does not join a list. The skew knob, where set, stands for the table; with
    // lists forced by their knob, a chunk whose variant is neither of the two takes the plain kernel.
    const long forced_skew = tuning().bulk_skew.load();
    auto list_pattern = [&](const ChunkRun& run) -> int {
        if (list_knob < 0 || !chunk_is_listable(K, run.n, es, run_aligned16(run), list_knob)) return -1;
        int skew = 0;
        if (forced_skew > 0) {
            skew = int(forced_skew);  // what a launch per chunk would run
        } else if (forced_skew == 0 && placement_query(run.in, K, run.out, es, &skew) != 2) {
            if (list_knob == 0) return -1;  // nothing recorded for these buffers
            skew = 0;
        }
        if (skew != 0 && skew != 3) return list_knob > 0 ? 0 : -1;
        // measured with pattern 3: sixteen inputs, 16 MiB chunks 5.94 -> 6.29 TB/s in list launches;
        // eight inputs, 25 MiB chunks 6.45 -> 6.17: those keep their launch per chunk
        if (skew == 3 && K <= 12 && list_knob == 0) return -1;
        return skew;
    };
    auto is_listable = [&](const ChunkRun& run) { return list_pattern(run) >= 0; };
    bool has_bulk = false;  // a launch that fills the GPU alone: bulk chunks and list launches
    size_t listable = 0;
    hfr_status st0 = walk([&](const ChunkRun& run) {
        if (is_bulk(run.n)) has_bulk = true;
        if (memo_status == HFR_OK && is_listable(run)) ++listable;
        return memo_status;
    });
    if (st0 != HFR_OK) return st0;
    const bool use_lists = listable >= 2;  // one chunk alone is an ordinary launch
    if (use_lists) has_bulk = true;
    enum { kBulk, kFold, kRingSingle, kStreamSingle, kList };
    // Batched launches stay on the caller's stream: a fork and a join of the
    // ring cost about 100 microseconds on this platform, more than the gaps
    // between a handful of batched launches (measured on 256 chunks of 64 KiB
    // to 4 MiB, 2 to 16 inputs: 0.06 to 12.5 microseconds per chunk on the
    // caller's stream against 0.36 to 13.3 dealt over four worker streams).
    const bool batches_on_ring = fold_knob == 1;
    auto classify = [&](const ChunkRun& run) {
        const size_t len = run.n;
        if (use_lists && is_listable(run)) return kList;
        if (is_bulk(len)) return kBulk;
        // beside a bulk launch only tiny chunks may run (see below)
        const bool leaves = has_bulk ? chunk_is_tiny(K, len, es) : chunk_gains_from_ring(K, len, es);
        if (fold && chunk_is_batchable(len, es) && (leaves || !has_bulk)) return kFold;
        return leaves && n_streams > 1 ? kRingSingle : kStreamSingle;
    };
    size_t folded = 0, ring_singles = 0;
    (void)walk([&](const ChunkRun& run) {
        const int c = classify(run);
        folded += c == kFold;
        ring_singles += c == kRingSingle;
        return HFR_OK;
    });

    // Folded chunks are split evenly over the fewest batched launches.
    const size_t cap = batch_capacity(K);
    const size_t batches = (folded + cap - 1) / cap;
    const size_t per_batch = batches ? (folded + batches - 1) / batches : cap;

    // Launches that leave the caller's stream go round the ring so that their
    // launch and ramp-up gaps overlap. A bulk chunk owns every compute unit
    // while it runs and depends on its workgroups moving in lock step: another
    // launch beside it (bulk or not) slows both down, and a hop to another
    // stream costs more than the gap it could hide, so bulk chunks stay in
    // order on the caller's stream, and in a call that has bulk chunks only
    // tiny chunks may run beside them. Mid-size chunks that fill the GPU on
    // their own stay on the caller's stream as well. The ring is forked only
    // when it has at least two launches to overlap.
    const size_t ring_launches = (batches_on_ring ? batches : 0) + ring_singles;
    const bool ring = n_streams > 1 && ring_launches > 1;
    StreamPool* pool = nullptr;
    int used = 1;
    if (ring) {
        used = ring_launches < size_t(n_streams) ? int(ring_launches) : n_streams;
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
    size_t next = 0;  // ring launches dealt so far
    auto ring_stream = [&]() { return ring ? pool_stream(pool, int(next++ % size_t(used))) : stream; };
    static thread_local ChunkBatch batch;
    batch.reset(per_batch, K);
    auto flush = [&]() -> hfr_status {
        if (batch.count == 0) return HFR_OK;
        hfr_status st = HFR_OK;
        hipStream_t s = batches_on_ring ? ring_stream() : stream;
        if (batch.count == 1) {
            st = enqueue_reduce(batch.items[0].in, K, batch.items[0].out, batch.items[0].n, dt, s);
        } else {
            const hipError_t e = dtype_ops(dt)->batched(batch.items.data(), batch.count, K, batch.aligned16, s);
            if (e != hipSuccess) st = fail_hip(e, "batched launch");
        }
        batch.count = 0;
        batch.aligned16 = true;
        return st;
    };
    // chunks for one bulk launch over a list
    static thread_local ChunkBatch list;
    const size_t list_cap = list_capacity(K);
    if (use_lists) list.reset(list_cap, K);
    // Nothing re-aligns the workgroups inside a launch, so a list launch is cut where a plain input
    // is cut into segments: at 128 MiB per buffer (64 MiB above twelve inputs).
    const size_t list_budget = (size_t(K > 12 ? 64 : 128) << 20) / es;  // elements per buffer and launch
    size_t list_elems = 0;
    int list_skew = 0;  // the variant of the chunks collected so far
    LaunchShape list_sh;
    int have_list_shape = -1;  // the variant list_sh was made for
    auto flush_list = [&]() -> hfr_status {
        if (list.count == 0) return HFR_OK;
        hfr_status st = HFR_OK;
        if (have_list_shape != list_skew) {
            st = list_shape(K, dt, list_skew, &list_sh);
            have_list_shape = st == HFR_OK ? list_skew : -1;
        }
        if (st == HFR_OK && list.count >= 2 && list_sh.grid != 0) {
            const hipError_t e = dtype_ops(dt)->list(list.items.data(), list.count, K, list_sh, stream);
            if (e != hipSuccess) st = fail_hip(e, "list launch");
        } else {
            for (size_t i = 0; i < list.count && st == HFR_OK; ++i)
                st = enqueue_reduce(list.items[i].in, K, list.items[i].out, list.items[i].n, dt, stream);
        }
        list.count = 0;
        list.aligned16 = true;
        list_elems = 0;
        return st;
    };
    result = walk([&](const ChunkRun& run) -> hfr_status {
        const int c = classify(run);
        if (c == kList) {
            const int pattern = list_pattern(run);
            if (list.count != 0 && (list_elems + run.n > list_budget || pattern != list_skew)) {
                const hfr_status st = flush_list();
                if (st != HFR_OK) return st;
            }
            list_skew = pattern;
            list.add(run.in, K, run.out, run.n);
            list_elems += run.n;
            return list.count == list_cap ? flush_list() : HFR_OK;
        }
        if (c == kFold) {
            batch.add(run.in, K, run.out, run.n);
            return batch.count == per_batch ? flush() : HFR_OK;
        }
        return enqueue_reduce(run.in, K, run.out, run.n, dt, c == kRingSingle ? ring_stream() : stream);
    });
    if (result == HFR_OK) result = flush_list();
    if (result == HFR_OK) result = flush();

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
    if (st != HFR_OK) return st;
    pool_unlock(pool);
    return noalloc_setup(nullptr);  // where this device's static chunk table lives
}

hfr_status hfr_shutdown(void) {
    placement_clear();
    return pool_destroy_all();
}

}  // extern "C"
