/*
 * Measurement helpers exported by liblutq.so next to the lutq_* entry points.  They are not part of
 * the method of the paper: they exist so that a benchmark can (a) quote the read bandwidth that a
 * plain streaming kernel reaches on the same device beside the nominal HBM peak, and (b) calibrate
 * the profiler's HBM byte counters against a copy of known size.
 */
#ifndef LUTQ_CALIB_H
#define LUTQ_CALIB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` (multiple of 16) from device memory `src` (16-byte aligned) with `grid` workgroups of
 * 256 threads and discards them. `sink4`: 4 writable device bytes. Asynchronous on `stream`.
 * Returns 0, 1 (bad argument) or 9 (launch failed). */
int lutq_calib_stream_read(const void* src, size_t bytes, int grid, void* sink4, void* stream);

/* Copies `bytes` (multiple of 16) from `src` to `dst` (device, 16-byte aligned, not overlapping).
 * Reads `bytes` and writes `bytes` of HBM traffic.  Same return codes. */
int lutq_calib_copy(const void* src, void* dst, size_t bytes, int grid, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LUTQ_CALIB_H */
