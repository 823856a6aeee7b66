/*
 * wfst_probe.h -- measured ceilings of the GPU the decoder runs on (C ABI).
 *
 * The decoder of wfst_decoder.h is irregular graph traversal; its roofline is quoted against the
 * published HBM bandwidth (cf. the paper's Section "Offline inference", whose throughput
 * discussion is in terms of how much work pruning leaves per frame).  These three probes say what
 * the chip delivers for the decoder's own access patterns, so that a fraction of the published
 * peak can be read next to a fraction of what is achievable.  Each call allocates its buffers on
 * the current device, runs on the default stream, synchronises and frees them.  Returns 0, or -1
 * on bad arguments or a HIP error.  All pointers are HOST memory.
 */
#ifndef WFST_PROBE_H_
#define WFST_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Plain device-to-device copy of `bytes` (>= 1 MiB) bytes, `reps` times back to back:
 * *gb_per_s = bytes read + bytes written per second, in GB/s. */
int32_t wfst_probe_copy(int64_t bytes, int32_t reps, double *gb_per_s);

/* `workgroups` workgroups of 1024 lanes; every lane reads 16 bytes from `loads_per_lane` (>= 8)
 * uniformly random 128-byte lines of a buffer of footprint_bytes (rounded down to a power of
 * two), 8 loads in flight per lane: *lines_per_s = line requests per second. */
int32_t wfst_probe_random_lines(int64_t footprint_bytes, int32_t workgroups, int32_t loads_per_lane,
                                double *lines_per_s);

/* The same with 64-bit atomicMin on uniformly random words, 4 in flight per lane:
 * *atomics_per_s = atomic operations per second. */
int32_t wfst_probe_atomics(int64_t footprint_bytes, int32_t workgroups, int32_t atomics_per_lane,
                           double *atomics_per_s);

#ifdef __cplusplus
}
#endif
#endif /* WFST_PROBE_H_ */
