/*
 * tsq_measure.h — measurement aids exported by the same library as tsq.h.  Nothing here is part of
 * the method: a benchmark uses these calls to time the kernels of one compress call one by one and
 * to find out what a kernel that only moves bytes reaches on the device at hand (the ceiling that
 * the achieved bandwidth of compress and restore is reported against, next to the published peak).
 * Conventions as in tsq.h: d_* are device pointers, `stream` is a hipStream_t passed as void*,
 * errors are return codes.
 */
#ifndef TSQ_MEASURE_H
#define TSQ_MEASURE_H

#include "tsq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * tsq_compress with every kernel of the call bracketed by HIP events on `stream`.  SYNCHRONIZES
 * `stream`.  ms_out (host, 4 floats) receives the kernels' durations in milliseconds: staged
 * pipeline {row statistics, scan, pack, 0}; single pass {the one kernel, 0, 0, 0}.  Same arguments
 * and result as tsq_compress otherwise.
 */
tsq_status tsq_compress_timed(const tsq_plan *plan, const void *d_in, void *d_blob, void *d_ws,
                              void *stream, float *ms_out);

/*
 * Copies `bytes` bytes (a multiple of 16; both pointers 16-byte aligned, regions disjoint) from d_src
 * to d_dst with one plain kernel: 16 bytes per lane, streaming loads and stores.  Enqueues only.
 */
tsq_status tsq_measure_copy(void *d_dst, const void *d_src, size_t bytes, void *stream);

/*
 * Reads `bytes` bytes (a multiple of 16, 16-byte aligned) with one plain kernel and writes (almost
 * always) nothing; d_sink points to 4 writable bytes.  Enqueues only.
 */
tsq_status tsq_measure_read(const void *d_src, size_t bytes, void *d_sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TSQ_MEASURE_H */
