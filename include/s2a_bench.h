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

/*
 * The same copy with the traffic shape of an activation kernel: besides the 16
 * bytes a lane moves from src to dst, it moves `side_bytes` (4 or 2: the packed
 * codes of 8 bf16 or 4 fp32 elements) to or from `side`, with the load / store
 * instructions the activation kernels use for their codes.
 *   side_is_input == 0   forward shape: src read, dst and side written
 *   side_is_input != 0   backward shape: src and side read, dst written
 * `side` holds nbytes/16 * side_bytes bytes, 4-byte aligned.  The benchmark times
 * it at an activation kernel's size as the measured ceiling of that kernel's
 * access pattern.  S2A_ERR_SIZE also for a side_bytes other than 2 or 4.
 */
int s2a_stream_copy_shaped(const void* src, void* dst, void* side, int64_t nbytes, int side_bytes,
                           int side_is_input, void* stream);

#ifdef __cplusplus
}
#endif

#endif /* S2A_BENCH_H */
