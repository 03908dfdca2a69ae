/*
 * rtams_measure.h - measurement aids of librtams.so.  NOT part of the method (arXiv 2408.02937) and not
 * needed to use the index: the benchmark and the profiling runs call them to time the list-scan kernel
 * inside a request and to calibrate hardware counters against kernels of known traffic.
 * Conventions as in rtams.h: d_* are device pointers, hip_stream is a hipStream_t passed as void*,
 * every function returns RTAMS_OK or a negative rtams_status.
 */
#ifndef RTAMS_MEASURE_H
#define RTAMS_MEASURE_H

#include "rtams.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measured duration of the list-scan kernel: with the parameter "profile_scan"
 * set to 1, every search brackets its scan launch with two HIP events on the
 * caller's stream; this call adds up the pairs of the requests that have
 * finished (ms_sum in milliseconds, launches = how many) and optionally resets
 * the sums.  Does not synchronise. */
int rtams_scan_time(rtams_index *ix, double *ms_sum, int64_t *launches, int reset);
/* Which kernel those timed launches were: launches3[0] counts the scans of the
 * vector unit (k_scan), [1] those on the matrix cores (k_scan_mm), [2] those
 * over product-quantiser codes (k_pq_scan), each since the last reset, counted
 * at launch while "profile_scan" is 1.  The library chooses per request. */
int rtams_scan_kernels(rtams_index *ix, int64_t *launches3, int reset);
/* A plain device-to-device copy kernel
 * (bytes a multiple of 16).  Profiler counters of HBM traffic are scaled by
 * what they read for this kernel, whose traffic is known. */
int rtams_copy_plain(void *d_dst, const void *d_src, size_t bytes, void *hip_stream);
/* A kernel that only reads `bytes`
 * (a multiple of 16) of device memory; d_sink points to 4 bytes of device
 * memory it may write.  Its rate is the practical ceiling a streaming read
 * reaches on the chip, reported beside the list scan's. */
int rtams_read_plain(const void *d_src, size_t bytes, float *d_sink, void *hip_stream);
#ifdef __cplusplus
}
#endif
#endif /* RTAMS_MEASURE_H */
