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

#include "lutq.h"

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

/* One launch of lutq_matmul_plan (same arguments, same result in Y; plan NULL = the default plan;
 * dtype 0 = fp16, 1 = bf16; M <= 4) through a measurement build of the kernel that also records where
 * the time of a launch goes: every wavefront reads the device's constant 100 MHz clock at eight points,
 *   0 wave started, 1 kernel arguments arrived, 2 first loads issued, 3 table built (barrier passed),
 *   4 first tile multiplied, 5 K loop done, 6 waves reduced, 7 outputs stored,
 * and writes them to trace[workgroup][wave][8] with 16 wave slots per workgroup (uint64, device memory,
 * 8-byte aligned, trace_bytes >= workgroups * 1024; slots of waves that do not exist stay untouched).  *workgroups receives the number of workgroups launched.
 * Measurement builds exist for 4-bit weights, group 64 or 128, plans with one or two row blocks per
 * wave and two tiles in flight; anything else returns 10 (plan).  Other return values are those of
 * lutq_matmul_plan (0 = launched; 7 = trace buffer too small).  Asynchronous on `stream`. */
int lutq_calib_matmul_trace(const void* X, const void* packed, const void* scales, const void* lut,
                            int bits, int group_size, int64_t M, int64_t N, int64_t K, int dtype,
                            void* Y, void* workspace, size_t workspace_bytes, void* stream,
                            const lutq_plan* plan, void* trace, size_t trace_bytes, int* workgroups);

#ifdef __cplusplus
}
#endif
#endif /* LUTQ_CALIB_H */
