/*
 * libhfr - the reduction arithmetic of the HFReduce allreduce on one MI355X.
 *
 * C ABI. Every pointer argument is marked HOST or DEVICE below. The library
 * never allocates device memory, never throws and never aborts: every entry
 * point returns an hfr_status. All buffers are owned by the caller.
 *
 * The operations follow the paper's statement of its allreduce (Section IV,
 * "HFReduce"): an intra-node reduce that sums the per-GPU copies of a gradient
 * chunk in GPU-index order (Algorithm 1), and an inter-node step that adds the
 * partial received from the neighbouring node to the local partial
 * (Algorithm 2, pass 1). Here the K per-GPU copies are K buffers resident in
 * one GPU's HBM.
 *
 * Arithmetic contract (identical for every entry point):
 *   - elements are widened exactly to IEEE-754 binary32;
 *   - every add and the scale multiply is ONE binary32 operation rounded to
 *     nearest-even on its own (never fused, never reassociated);
 *   - the K-way sum is taken left to right: ((in[0] + in[1]) + in[2]) + ...;
 *   - bf16 / fp16 / fp8 results are rounded once, to nearest-even, when stored;
 *   - subnormals are honoured (no flush); a NaN input gives a NaN output whose
 *     payload and sign are unspecified.
 * Results are therefore reproducible bit for bit, independent of n, of the
 * chunking and of the launch shape.
 *
 * Threads: entry points may be called from several host threads at once (on
 * different streams, or on one stream in whatever order the calls are made);
 * the worker streams of hfr_reduce_buckets are shared per device, so calls that
 * fork them take turns. The tuning knobs are process-wide.
 */
#ifndef HFR_H_
#define HFR_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same declaration as the HIP runtime's; repeating it keeps this header usable
 * from plain C without the HIP headers. */
typedef struct ihipStream_t* hipStream_t;

typedef enum {
    HFR_OK = 0,
    HFR_ERR_INVALID_ARG = 1,       /* null pointer with n > 0, K out of range, zero chunk size ... */
    HFR_ERR_UNSUPPORTED_DTYPE = 2, /* dtype code not listed in hfr_dtype */
    HFR_ERR_MISALIGNED = 3,        /* a pointer is not aligned to its element size */
    HFR_ERR_OVERLAP = 4,           /* the output partially overlaps an input */
    HFR_ERR_HIP = 5                /* a HIP runtime call failed; text via hfr_last_error() */
} hfr_status;

/* Element types: the four the paper lists for the reduction (Section IV-D.1:
 * FP32 / FP16 / BF16 / FP8). The narrow types are widened exactly, accumulated
 * in binary32 and rounded once, to nearest even, when stored; subnormals are
 * kept. fp16 is IEEE binary16; fp8 is either OCP format: E4M3 (bias 7, no
 * infinity, largest number 448, NaN = S.1111.111) or E5M2 (bias 15, IEEE-like).
 * A result that does not fit becomes infinity where the type has one (bf16,
 * fp16, E5M2) and NaN where it has none (E4M3); nothing saturates. */
typedef enum {
    HFR_F32 = 0,
    HFR_BF16 = 1,
    HFR_F16 = 2,
    HFR_FP8_E4M3 = 3,
    HFR_FP8_E5M2 = 4
} hfr_dtype;

#define HFR_MAX_K 16       /* most input buffers per reduction */
#define HFR_MAX_STREAMS 16 /* most worker streams hfr_reduce_buckets will use */

/*
 * K-way elementwise sum: the inner loop of Algorithm 1, which adds every
 * GPU's copy of one chunk, in GPU-index order, into the node's chunk buffer.
 *
 *   out[i] = (((in[0][i] + in[1][i]) + in[2][i]) + ...) + in[K-1][i],  0 <= i < n
 *
 * in      HOST array of K DEVICE pointers, each to n contiguous elements of
 *         type dt. Read during the call only (the pointers are copied into the
 *         kernel arguments); the caller may free the array on return.
 * K       1 <= K <= HFR_MAX_K. K == 1 is a copy.
 * out     DEVICE pointer to n elements of type dt. May be exactly equal to one
 *         of in[j] (the paper's form is in place). Any other overlap between
 *         out and an input is rejected with HFR_ERR_OVERLAP.
 * n       element count, any value (no multiple-of-vector requirement).
 *         n == 0 returns HFR_OK and enqueues nothing.
 * stream  the work is enqueued on this stream (0 = the null stream) and the
 *         call returns without waiting for it.
 *
 * Pointers need only element alignment; when all K+1 are 16-byte aligned the
 * fully vectorised path is taken. Argument errors are detected on the host
 * before anything is enqueued.
 */
hfr_status hfr_reduce_sum(const void* const* in, int K, void* out, size_t n, hfr_dtype dt,
                          hipStream_t stream);

/*
 * Two-operand combine and average: Algorithm 2, pass 1 (the partial received
 * from the neighbouring node is added into the local one), with the averaging
 * factor of the data-parallel allreduce applied once afterwards.
 *
 *   out[i] = fl( fl(a[i] + b[i]) * scale )
 *
 * a, b    DEVICE pointers to n elements of type dt (local partial, received
 *         remote partial).
 * out     DEVICE pointer to n elements; may be exactly equal to a or b.
 * scale   binary32 multiplier (e.g. 1 / (GPUs per node * nodes)); 1.0f gives
 *         the plain sum bit for bit.
 * Other conventions as for hfr_reduce_sum.
 */
hfr_status hfr_combine_avg(const void* a, const void* b, void* out, size_t n, float scale,
                           hfr_dtype dt, hipStream_t stream);

/*
 * K-way sum with the averaging factor folded in, for an allreduce without an
 * inter-node stage (Algorithm 1 alone, then the data-parallel mean):
 *
 *   out[i] = narrow( fl( (((in[0][i] + in[1][i]) + ...) + in[K-1][i]) * scale ) )
 *
 * The fp32 sum is NOT rounded to the storage type before the multiply, so for
 * bf16 this is its own function, not hfr_reduce_sum followed by a scaling pass
 * (it saves that pass's 2 * n * s bytes). scale = 1.0f gives hfr_reduce_sum bit
 * for bit. Arguments as for hfr_reduce_sum.
 */
hfr_status hfr_reduce_avg(const void* const* in, int K, void* out, size_t n, float scale, hfr_dtype dt,
                          hipStream_t stream);

/*
 * Intra-node sum and inter-node combine in one pass over memory: Algorithm 1
 * reduces chunk i inside the node and hands it straight to the inter-node
 * step, which adds the partial received from the neighbouring node
 * (Algorithm 2, pass 1). When that partial is already there,
 * both happen in one kernel:
 *
 *   p      = narrow( ((in[0][i] + in[1][i]) + ...) + in[K-1][i] )   (the node partial, as stored)
 *   out[i] = narrow( fl( fl( widen(p) + remote[i] ) * scale ) )
 *
 * Bit for bit the result of hfr_reduce_sum followed by hfr_combine_avg, but the
 * node partial never travels to HBM and back: (K + 2) * n * s bytes instead of
 * (K + 4) * n * s. 1 <= K <= HFR_MAX_K - 1. `remote` is a DEVICE pointer to n
 * elements; out may be exactly equal to remote or to one of in[j].
 */
hfr_status hfr_reduce_combine_avg(const void* const* in, int K, const void* remote, void* out, size_t n,
                                  float scale, hfr_dtype dt, hipStream_t stream);

/*
 * Slice-only K-way sum: the shape of the paper's HFReduce-with-NVLink variant
 * (Section IV-C), where every GPU of a group first reduces its own part of the
 * data. [0, n) is cut into `world` contiguous slices whose lengths differ by
 * at most one (the first n % world slices are the longer ones); only slice
 * `rank` is reduced:
 *
 *   out[i] = in-order K-way sum of in[j][i]   for begin <= i < end
 *
 * in[j] and out point to the FULL n-element buffers; elements of out outside
 * the slice are not touched. 0 <= rank < world. hfr_slice_bounds (host only,
 * touches no device) returns [begin, end) of a slice, or the empty range 0, 0
 * for a rank / world pair that names no slice.
 */
hfr_status hfr_reduce_scatter_slice(const void* const* in, int K, void* out, size_t n, int rank, int world,
                                    hfr_dtype dt, hipStream_t stream);
void hfr_slice_bounds(size_t n, int rank, int world, size_t* begin, size_t* end);

/*
 * Broadcast: Algorithm 2, pass 2 - the reduced chunk is copied to every GPU
 * of the node, one copy per GPU. Here: one read of
 * src, K writes (K separate copies would read src K times).
 *
 *   dst[j][i] = src[i]    for 0 <= j < K, 0 <= i < n      (an exact copy)
 *
 * src   DEVICE pointer to n elements of type dt.
 * dst   HOST array of K DEVICE pointers to n elements each (read during the
 *       call only). A dst[j] may be exactly equal to src or to another dst[i];
 *       any other overlap is rejected with HFR_ERR_OVERLAP.
 * Other conventions as for hfr_reduce_sum. (The paper's general reduce operation is
 * hfr_reduce_sum itself.)
 */
hfr_status hfr_broadcast(const void* src, void* const* dst, int K, size_t n, hfr_dtype dt,
                         hipStream_t stream);

/* One gradient bucket: K input buffers and one output buffer of n elements. */
typedef struct {
    const void* const* in; /* HOST array of K DEVICE pointers */
    void* out;             /* DEVICE pointer */
    size_t n;              /* elements */
} hfr_bucket;

/*
 * Chunked, pipelined reduction of a list of gradient buckets: Algorithm 1's
 * outer structure (the data is cut into chunks of the paper's Chunk_Size and
 * reduced chunk after chunk), fed by the stream of gradient buckets a
 * data-parallel backward pass produces (Section V-A). Every bucket is cut into
 * chunks of chunk_elems elements (the last chunk of a bucket may be shorter)
 * and every chunk is reduced with the arithmetic of hfr_reduce_sum; the result
 * is bit-identical to hfr_reduce_sum on each whole bucket.
 *
 * Chunks that follow each other in memory - every input and the output of the
 * next chunk start where the previous chunk's end, as the chunks of one bucket
 * and buckets cut from one flat gradient buffer do - are one longer elementwise
 * sum and are handled as ONE chunk of the summed length (the bits are the same;
 * a run stops where an input and the output would start to overlap partially).
 * For a gradient that is contiguous per peer the chunk loop therefore costs
 * nothing: 256 chunks of 64 KiB run as one launch, and multi-GiB gradients as
 * equal launches of at most 128 MiB per buffer (worth about 3 % against one
 * launch per 50 MiB bucket).
 *
 * Where a chunk (after that merging) runs, by its size; "traffic" = K reads +
 * 1 write:
 *   - up to 8 MiB per buffer: folded, with its neighbours in list order, into
 *     batched launches on `stream` (one grid over about 3800 / (8 * (K + 3))
 *     chunks, the chunk table in the kernel arguments), because a launch per
 *     chunk costs the host more than such a chunk runs for;
 *   - larger, up to 96 MiB of traffic: a launch of its own, dealt round-robin
 *     over the worker streams so that launch and ramp-up gaps overlap;
 *   - with 8 or 16 inputs and 16-byte aligned buffers, 10 to 32 MiB per buffer
 *     (16 inputs: 5 to 24 MiB), on buffers for which the placement table has
 *     recorded the plain kernel (pattern 0; see hfr_tune_placement) or, with
 *     16 inputs, pattern 3: together
 *     with the other such chunks of the call in bulk launches over a list of
 *     chunks on `stream` (up to 128 MiB per buffer and launch, chunk table in
 *     the kernel arguments), which keeps the chip busy across chunk
 *     boundaries: 2 to 10 % over a launch per chunk;
 *   - larger still ("bulk" launch shape, from tens of MiB per buffer; it fills
 *     the GPU alone): in list order on `stream`, cut like any long input.
 * In a call that contains bulk chunks nothing but chunks of at most 16 MiB of
 * traffic leaves `stream` or is folded: a mid-size launch beside a bulk launch
 * slows both.
 *
 * buckets     HOST array of n_buckets descriptors (read during the call only).
 * chunk_elems > 0. A value >= a bucket's n means one launch for that bucket.
 * n_streams   1 <= n_streams <= HFR_MAX_STREAMS (an upper bound on the worker
 *             streams used). With 1, or with fewer than two launches for the
 *             worker streams, everything is enqueued directly on `stream`. Otherwise the
 *             library's own worker streams fork from `stream` (they wait for
 *             everything already enqueued on it) and join back into it, so
 *             the caller sees ordinary stream order: work enqueued on
 *             `stream` afterwards runs after every chunk. The host is never
 *             blocked.
 * All buckets are validated before the first chunk is enqueued. Output
 * buffers of different buckets must not overlap each other or another bucket's
 * inputs (not checked).
 * The worker streams are created on first use for the current device, at
 * default priority, and kept until hfr_shutdown().
 */
hfr_status hfr_reduce_buckets(const hfr_bucket* buckets, size_t n_buckets, int K, hfr_dtype dt,
                              size_t chunk_elems, int n_streams, hipStream_t stream);

/*
 * The same reduction of a bucket list with the fewest launches: small buckets
 * (up to 8 MiB per buffer) are folded, in list order, into batched launches
 * whose bucket table (K + 1 pointers and a size per bucket) travels in the
 * kernel arguments - no device allocation, no copy; about 3800 / (8 * (K + 3))
 * buckets per launch. Larger buckets get a launch of their own. Everything is
 * enqueued on `stream` in list order. For lists of many small buckets this
 * removes the per-launch host cost (a few microseconds each); it is the fold
 * that hfr_reduce_buckets applies to its small chunks, as an entry point of
 * its own for callers whose buckets are already cut. Results are bit-identical
 * to hfr_reduce_sum on each bucket. Validation and conventions as for
 * hfr_reduce_buckets.
 */
hfr_status hfr_reduce_buckets_batched(const hfr_bucket* buckets, size_t n_buckets, int K, hfr_dtype dt,
                                      hipStream_t stream);

/*
 * One chunk of a chunk table that lives in DEVICE memory. Only the first K
 * input pointers are read.
 */
typedef struct {
    const void* in[HFR_MAX_K]; /* DEVICE pointers */
    void* out;                 /* DEVICE pointer */
    size_t n;                  /* elements; 0 = nothing to do */
} hfr_chunk;

/*
 * The K-way sum of hfr_reduce_sum for every chunk of a table in DEVICE memory
 * (Algorithm 1's chunk loop with the chunk list itself on the GPU): ONE launch
 * whatever the number of chunks, and since the host never reads the table it
 * may be written by work enqueued earlier on `stream` - a copy, or a kernel
 * that produces chunks. This is the latency-regime end of the bucket entry
 * points: hfr_reduce_buckets and hfr_reduce_buckets_batched pay one launch per
 * few dozen small chunks, this one a single launch.
 *
 * table             DEVICE array of n_chunks entries, 8-byte aligned. It must
 *                   stay unchanged until the launch has run.
 * chunk_elems_hint  > 0: the usual chunk length, used to size the launch only;
 *                   chunks of any length (longer or shorter) are summed in full.
 * Because the table is not visible to the host nothing in it can be checked:
 * every chunk must satisfy what hfr_reduce_sum would have checked (pointers
 * aligned to the element size, out equal to an input or not overlapping any,
 * n elements readable and writable). 16-byte alignment is detected per chunk
 * on the device. Results are bit-identical to hfr_reduce_sum on each chunk.
 */
hfr_status hfr_reduce_chunk_table(const hfr_chunk* table, size_t n_chunks, size_t chunk_elems_hint, int K,
                                  hfr_dtype dt, hipStream_t stream);

/*
 * hfr_reduce_chunk_table for callers that cannot allocate device memory for
 * the table: code that runs under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. The chunk list is a HOST array here; the
 * library stages it in a static device array of its own (HFR_NOALLOC_MAX_CHUNKS
 * entries of sizeof(hfr_chunk) = 144 bytes, 576 KiB per GPU, held until the
 * process ends) with small fill launches that carry the entries in their
 * kernel arguments, then sums every chunk with ONE launch of the same kernel
 * hfr_reduce_chunk_table uses. It calls no allocator and makes no copy from
 * host memory: `chunks` is read during the call only.
 *
 * chunks            HOST array of n_chunks entries (DEVICE pointers inside).
 *                   Being on the host, every entry gets the checks of
 *                   hfr_reduce_sum before anything is enqueued.
 * n_chunks          at most HFR_NOALLOC_MAX_CHUNKS, else HFR_ERR_INVALID_ARG
 *                   (hfr_last_error() names the limit).
 * chunk_elems_hint, K, dt, stream   as hfr_reduce_chunk_table.
 * Every call on a GPU uses that GPU's one static table: calls on the same
 * stream follow each other safely, calls that may overlap in time on one GPU
 * (different streams, different host threads) race on it and must be
 * serialised by the caller. Results are bit-identical to
 * hfr_reduce_chunk_table on the same chunks.
 */
#define HFR_NOALLOC_MAX_CHUNKS 4096
hfr_status hfr_reduce_chunks_noalloc(const hfr_chunk* chunks, size_t n_chunks, size_t chunk_elems_hint, int K,
                                     hfr_dtype dt, hipStream_t stream);

/* Optional: create the worker streams and events of the current device ahead
 * of the first hfr_reduce_buckets call, and look up the device address of the
 * static table of hfr_reduce_chunks_noalloc. Idempotent. */
hfr_status hfr_init(void);

/* Destroy the worker streams and events of every device. The caller must have
 * synchronised its streams first. Idempotent. */
hfr_status hfr_shutdown(void);

/* Static text for a status code (never NULL). */
const char* hfr_status_string(hfr_status s);

/* Text of the most recent HIP failure (or exceeded library limit) on the
 * calling thread ("" if none). The pointer stays valid until the thread's next
 * failing call. */
const char* hfr_last_error(void);

/* Version: major * 10000 + minor * 100 + patch. */
int hfr_version(void);

/*
 * Placement tuning. How fast K buffers stream together depends on how far
 * apart they lie: at some distances the K loads of one offset fall into the
 * same DRAM bank and the bulk launch shape loses up to 12 % of its bandwidth.
 * The bulk kernels exist in "skewed" variants in which some streams run a few
 * MiB ahead of the others (same operands, same order, same bits): three
 * patterns for 8 and 9 inputs, with every epilogue; pattern 3 alone, for the
 * plain sum, for the other input counts of the bulk shape (5 to 16).
 * Which variant is fastest is a property of the placement - the
 * distances of in[1..K-1] and of out from in[0], the element size and the
 * device - and is found by measurement, in one of two ways:
 *
 *   on the fly (default)  the first bulk launches on a placement the library
 *       has not seen run the plain kernel and the variants that exist for K
 *       inputs in turn (three launches each: twelve for 8 and 9 inputs, six
 *       otherwise), each between two events on the caller's stream; a later launch
 *       finds those events finished and records the fastest variant. The host
 *       never blocks, results are the same bits throughout, and launches on a
 *       stream that is being captured into a graph take no trials.
 *   hfr_tune_placement    the explicit form: times those kernels on the
 *       caller's buffers (four launches each) and records the fastest
 *       before it returns. Unlike every other entry point it BLOCKS the host
 *       until its launches on `stream` have finished.
 *
 * Every later K-way call (hfr_reduce_sum, _avg, _combine_avg with the remote
 * partial as input K, _scatter_slice, the bucket entry points) whose buffers
 * lie at the same distances - the same buffers, or chunks, slices and segments
 * of them at a common offset - uses the recorded variant where it exists for
 * that call's K and epilogue, the plain kernel otherwise. The table holds 64
 * placements per process (the oldest is replaced) and is emptied by
 * hfr_shutdown().
 *
 * in, K, out, n, dt   as hfr_reduce_sum; `out` receives the K-way sum (it is
 *                     written four times per kernel tried) and must not be one of the
 *                     inputs (HFR_ERR_INVALID_ARG).
 * chosen              HOST pointer or NULL: the pattern recorded, 0 (plain) to 3.
 * Inputs that do not take the bulk shape (too small, fewer than 5 inputs, not
 * 16-byte aligned) are summed once, nothing is recorded and *chosen is 0.
 */
hfr_status hfr_tune_placement(const void* const* in, int K, void* out, size_t n, hfr_dtype dt,
                              hipStream_t stream, int* chosen);

/*
 * What the placement table holds for these buffers (host only, enqueues
 * nothing): *state = 0 unknown, 1 being measured on the fly, 2 recorded;
 * *pattern = the recorded variant, 0 (plain) to 3, and 0 while nothing is
 * recorded. in is a HOST array of K DEVICE pointers; state and pattern are
 * HOST pointers and may be NULL.
 */
hfr_status hfr_placement_query(const void* const* in, int K, const void* out, hfr_dtype dt, int* state,
                               int* pattern);

/*
 * Placement hint for callers that own the memory the K buffers live in (a
 * staging arena for the peers' gradients, a flat gradient buffer per peer):
 * the distance in bytes at which to carve the K inputs and the output, one
 * after the other, from ONE device allocation so that the K + 1 streams of a
 * reduction fall into different DRAM banks and channels. Buffers that a general
 * allocator places independently land in a good or a bad class by chance
 * (K = 8 bf16, 128 MiB per buffer: 6.46 to 6.85 TB/s from process to process);
 * at this stride the same kernel runs at 6.8 TB/s every time, and the placement
 * table has nothing to repair. The result is at least bytes_per_buffer, a
 * multiple of 2 MiB, and less than 16 MiB above it. A rule fitted to
 * measurements on this GPU (see the definition); host only, touches no device.
 * Returns 0 if the size is too large to round up.
 */
size_t hfr_peer_stride(size_t bytes_per_buffer);

/*
 * The measured form of hfr_peer_stride, for callers that have their arena
 * already: times the K-way sum of K + 1 buffers of n elements carved from
 * `arena` at nine candidate distances (the size rounded up to 2 MiB plus 0 to
 * 14 MiB, and hfr_peer_stride's value) and returns the fastest in *stride; the
 * rule's value is kept unless another beats it by more than 1.5 %. Where the
 * rule misses (it is a fit: K = 8 at 1500 MiB per buffer it gives 1512 MiB,
 * 6.33 TB/s, where 1500 runs at 6.51) this finds the better distance.
 *
 * arena, arena_bytes  DEVICE memory, 16-byte aligned, at least
 *                     K * hfr_peer_stride(n * elem) + n * elem bytes
 *                     (HFR_ERR_INVALID_ARG if smaller); candidates that do not
 *                     fit are skipped. Its contents are read as they are and
 *                     OVERWRITTEN where candidate outputs lie.
 * K, n, dt            as hfr_reduce_sum; at most 256 MiB per buffer are timed.
 * stride              HOST pointer, required: the distance in bytes.
 * Like hfr_tune_placement it BLOCKS the host until its launches on `stream`
 * (a few dozen) have finished. Allocates nothing.
 */
hfr_status hfr_tune_peer_stride(void* arena, size_t arena_bytes, int K, size_t n, hfr_dtype dt,
                                hipStream_t stream, size_t* stride);

/*
 * What the HIP runtime reports for the current device, for the bandwidth
 * figures a benchmark prints beside its measurements: number of compute units,
 * memory clock in kHz and memory bus width in bits (reported peak bandwidth =
 * 2 * clock * width / 8 for double-data-rate memory). Each pointer is a HOST
 * pointer and may be NULL; a value the runtime does not report is set to 0.
 * Returns HFR_ERR_HIP when no device can be queried.
 */
hfr_status hfr_device_info(int* compute_units, int* memory_clock_khz, int* memory_bus_bits);

/*
 * Launch-shape knobs, for benchmarking. They never change results.
 * Two launch shapes exist: "wide" (many workgroups, for small and medium
 * inputs) and "bulk" (one workgroup per compute unit walking the buffers in
 * lock step with deferred store bursts, for large inputs).
 *   HFR_TUNE_GRID_CAP        wide: most workgroups per launch (0 = default:
 *                            one per tile, however many that makes)
 *   HFR_TUNE_UNROLL          wide: 16-byte vectors per lane per trip: 1, 2, 4
 *                            (0 = default)
 *   HFR_TUNE_BULK_GRID       bulk: workgroups per launch (0 = one per
 *                            compute unit)
 *   HFR_TUNE_BULK_MIN_BYTES  bytes per buffer from which the bulk shape is
 *                            used, for any K (0 = default rule, which also
 *                            looks at K; -1 = never). Buffers that are not
 *                            16-byte aligned always take the wide shape.
 *   HFR_TUNE_BULK_SKEW       bulk: stream skew pattern 1, 2 or 3 for every
 *                            launch that has it (8 and 9 inputs: all three;
 *                            5 to 16 inputs, plain sum: pattern 3; any other
 *                            launch runs the plain kernel). 0 = the pattern
 *                            the placement table holds for the buffers,
 *                            measured on the fly where it holds none;
 *                            -1 = never skew
 *   HFR_TUNE_PLACEMENT_ONLINE  0 = placements the table does not hold are
 *                            measured on the fly (default), -1 = they run the
 *                            plain kernel until hfr_tune_placement is called
 *   HFR_TUNE_SEGMENT_MIB     inputs longer than this many MiB per buffer are
 *                            cut into back-to-back launches of that length
 *                            (0 = default rule, which looks at K; 1 .. 65536)
 *   HFR_TUNE_BUCKET_FOLD    hfr_reduce_buckets: 0 = adjacent chunks are merged
 *                            and small chunks folded into batched launches on
 *                            the caller's stream
 *                            (default), 1 = the same with the batched launches
 *                            dealt over the worker streams, -1 = one launch
 *                            per chunk on the worker streams (the two
 *                            schedules the default is measured against)
 *   HFR_TUNE_BULK_BLOCK      bulk K-way sum: lanes per workgroup, a multiple of
 *                            32 from 64 to 384 (0 = the measured table, by
 *                            element type and K; values above what the kernel
 *                            for that K was built for are clamped)
 *   HFR_TUNE_BULK_PACE       bulk K-way sum: pause after each trip of a
 *                            workgroup, in units of 64 clocks, 1 .. 64
 *                            (0 = the measured table, -1 = no pause)
 *   HFR_TUNE_WIDE_WGS_PER_CU wide and batched K-way sum: most workgroups
 *                            resident on one compute unit at a time, 1 .. 16
 *                            (0 = default rule by input count and size: none
 *                            for small inputs and for two operands, two to
 *                            four otherwise; -1 = never a limit)
 *   HFR_TUNE_BUCKET_LIST    hfr_reduce_buckets, 8 or 16 inputs: 0 = chunks of
 *                            10 to 32 MiB per buffer (16 inputs: 5 to 24)
 *                            that lie apart, on placements recorded as
 *                            pattern 0 (16 inputs: or 3), run together as
 *                            bulk launches over a list of chunks
 *                            (default), 1 = every 16-byte aligned chunk does,
 *                            whatever its size, -1 = never (the two schedules
 *                            the default is measured against)
 * HFR_TUNE_BULK_GRID and HFR_TUNE_BULK_MIN_BYTES also steer the bulk shape of
 * hfr_broadcast (three or more destinations).
 * Returns HFR_ERR_INVALID_ARG for an unknown knob or value. Also read once from
 * the environment (HFR_GRID_CAP, HFR_UNROLL, HFR_BULK_GRID, HFR_BULK_MIN_BYTES,
 * HFR_BULK_SKEW, HFR_BUCKET_FOLD, HFR_PLACEMENT_ONLINE, HFR_SEGMENT_MIB,
 * HFR_BULK_BLOCK, HFR_BULK_PACE, HFR_WIDE_WGS_PER_CU, HFR_BUCKET_LIST).
 */
typedef enum {
    HFR_TUNE_GRID_CAP = 0,
    HFR_TUNE_UNROLL = 1,
    HFR_TUNE_BULK_GRID = 2,
    HFR_TUNE_BULK_MIN_BYTES = 3,
    HFR_TUNE_BULK_SKEW = 4,
    HFR_TUNE_BUCKET_FOLD = 5,
    HFR_TUNE_PLACEMENT_ONLINE = 6,
    HFR_TUNE_SEGMENT_MIB = 7,
    HFR_TUNE_BULK_BLOCK = 8,
    HFR_TUNE_BULK_PACE = 9,
    HFR_TUNE_WIDE_WGS_PER_CU = 10,
    HFR_TUNE_BUCKET_LIST = 11
} hfr_tune_knob;
hfr_status hfr_set_tuning(hfr_tune_knob knob, long value);

#ifdef __cplusplus
}
#endif
#endif /* HFR_H_ */
