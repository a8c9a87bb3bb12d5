/*
 * libhfr_probe - streaming probes for the benchmark's "ceilings" table.
 *
 * Not part of the reduction library: these kernels compute nothing of the
 * paper's method. They move bytes in the same access shapes as libhfr's
 * kernels (R read streams, W write streams, 16-byte vectors, non-temporal) so
 * that a benchmark can put measured HBM ceilings - read-only, fill-only, copy,
 * 2 reads : 1 write, 8 reads : 1 write - beside the kernels' own figures
 * (the paper's bytes model, Section IV-D.3, counts the same reads and writes).
 * C ABI; every pointer argument is marked HOST or DEVICE.
 */
#ifndef HFR_PROBE_H_
#define HFR_PROBE_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t* hipStream_t;

#define HFR_PROBE_MAX_STREAMS 16

/* Launch shapes, as in libhfr: many workgroups with a grid-stride loop, or one
 * workgroup per compute unit walking the buffers in lock step with its results
 * parked in registers and stored in bursts. */
typedef enum { HFR_PROBE_WIDE = 0, HFR_PROBE_BULK = 1 } hfr_probe_shape;

/*
 * One streaming pass: every 16-byte vector position of nbytes is read from each
 * of the n_read buffers, the vectors are XORed (no floating point), and the
 * result is written to each of the n_write buffers. n_write == 0 is a
 * read-only pass: the XOR is stored to `sink` only if it equals a pattern that
 * the caller's data does not contain (so that the loads cannot be elided);
 * n_read == 0 is a fill of the value 0.
 *
 * rd      HOST array of n_read DEVICE pointers (0 <= n_read <= 16), each to
 *         nbytes readable bytes, 16-byte aligned.
 * wr      HOST array of n_write DEVICE pointers (0 <= n_write <= 16), each to
 *         nbytes writable bytes, 16-byte aligned. Supported pairs:
 *         n_write <= 1 with any n_read, or n_read <= 1 with any n_write.
 * sink    DEVICE pointer to at least 16 writable bytes (read-only passes).
 * nbytes  a multiple of 32 KiB (eight 16-byte vectors for each of 256 lanes).
 * Returns 0 on success, 1 for an argument that is out of range, 5 for a HIP
 * failure. Only enqueues; completion is ordered on `stream`.
 */
int hfr_probe_stream(const void* const* rd, int n_read, void* const* wr, int n_write, void* sink, size_t nbytes,
                     hfr_probe_shape shape, hipStream_t stream);

/*
 * The bulk shape of hfr_probe_stream with the two knobs libhfr's bulk kernels
 * have for the number of loads a compute unit keeps in flight: `lanes` per
 * workgroup (a multiple of 32 from 64 to 384; a tile is lanes * U vectors,
 * with U the vectors per lane and trip that the stream count implies) and a
 * pause of `pace` * 64 clocks (0 .. 64) after each trip. Whole tiles only:
 * the last nbytes mod (tile size) bytes of each buffer are not touched.
 * Other arguments and the return value as above.
 */
int hfr_probe_stream_paced(const void* const* rd, int n_read, void* const* wr, int n_write, void* sink, size_t nbytes,
                           int lanes, int pace, hipStream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* HFR_PROBE_H_ */
