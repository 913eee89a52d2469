/*
 * stream_copy.h - a plain device copy kernel of known traffic, built into its own
 * small library (libmaddness_calib.so).  It is NOT part of the MADDNESS method or of
 * libmaddness: the benchmark uses it to quote a copy rate beside its own figures, and
 * the profiler summaries use it to scale the memory counters (a launch reads `bytes`
 * and writes `bytes`).
 */
#ifndef MADDNESS_CALIB_STREAM_COPY_H
#define MADDNESS_CALIB_STREAM_COPY_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Copies `bytes` bytes (a multiple of 16; both DEVICE pointers 16-byte aligned) from
 * src to dst with a grid-stride kernel of non-temporal 16-byte loads and stores on
 * `stream` (a hipStream_t; NULL: the null stream).  Returns 0, -1 for a null pointer,
 * -3 for a misaligned pointer or size, -4 if the launch was refused.
 */
int calib_stream_copy(const void *src, void *dst, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
