/*
 * signvote_bench.h -- measurement helper exported by libsignvote next to the API of signvote.h.
 *
 * Not part of the method: a plain streaming copy used (a) as the yardstick for what HBM sustains on
 * this GPU for a 1:1 read/write stream, next to which the library's kernels are reported, and (b) as
 * the kernel of known traffic that scales the profiler's FETCH_SIZE / WRITE_SIZE counters.
 */
#ifndef SIGNVOTE_BENCH_H
#define SIGNVOTE_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * dst[0 .. bytes) <- src[0 .. bytes), device memory, non-overlapping, both 16-byte aligned, bytes a
 * positive multiple of 16.  One 16-byte non-temporal load and store per thread.  Asynchronous on
 * `stream` (hipStream_t as void*, NULL = default stream).  Returns 0, or the negative ssv_status
 * codes of signvote.h (NULL pointer -1, bad size -2, misaligned -3, launch failure -6).
 */
int ssv_bench_copy(const void* src, void* dst, int64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SIGNVOTE_BENCH_H */
