/*
 * s2a_bench.h -- measurement aids exported by libs2a.so next to the method's
 * entry points (include/s2a.h).  Nothing here is part of the activation path:
 * the benchmark uses it to measure what the memory system sustains for the
 * access pattern of the activation kernels.  Return codes are those of s2a.h.
 */
#ifndef S2A_BENCH_H
#define S2A_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A plain streaming copy of `nbytes` bytes (a multiple of 16; src and dst
 * device, 16-byte aligned, not overlapping) with the launch shape and the load /
 * store instructions of the activation kernels -- one 16-byte vector per lane,
 * single-wave blocks.  S2A_ERR_SIZE if nbytes is negative or not a multiple of
 * 16, S2A_ERR_ALIGN for misaligned pointers.
 */
int s2a_stream_copy(const void* src, void* dst, int64_t nbytes, void* stream);

#ifdef __cplusplus
}
#endif

#endif /* S2A_BENCH_H */
