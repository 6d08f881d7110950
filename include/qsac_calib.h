/*
 * qsac_calib.h - measurement aids for the QSAC benchmark (libqsac_calib.so).
 *
 * Two kernels of known size that the benchmark and the profiler summaries are held against.  They are
 * not part of the QSAC step and are kept out of libqsac.so.  Both functions only enqueue; they return
 * 0 on success, -2 for a NULL pointer, -7 for a misaligned pointer or size, -5 if the launch failed.
 */
#ifndef QSAC_CALIB_H
#define QSAC_CALIB_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues a plain device-to-device copy of `bytes` bytes (a multiple of 16, both pointers DEVICE and
 * 16-byte aligned) on `stream` (hipStream_t, NULL = default stream).  It reads `bytes` and writes
 * `bytes`, which is what profiler memory counters are scaled against.
 */
int qsac_calibration_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Enqueues a kernel that only reads `bytes` bytes (a multiple of 16) at DEVICE pointer `src` (16-byte
 * aligned) on `stream`: 2048 workgroups, a contiguous span each, eight 16-byte loads per thread in flight.
 * Its duration is what a launch of that size can reach on the part with no arithmetic at all.  `sink` is a
 * DEVICE u32 (4-byte aligned) that is (practically never) written; it keeps the loads alive.
 */
int qsac_calibration_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QSAC_CALIB_H */
