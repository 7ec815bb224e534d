/*
 * signvote_qsgd.h -- the comparison compressors of the paper, exported by libsignvote next to signvote.h:
 * ternary ("1-bit") QSGD with the Euclidean norm ("L2 QSGD") or the largest magnitude ("max QSGD"), as Appendix B
 * ("Bits sent per iteration") defines them and as the QSGD figure of Section 4 uses them in the 1-way scheme.
 *
 *     norm_m    = ||g_m||_2  or  ||g_m||_inf                                       (ssv_qsgd_norms)
 *     q_m[i]    = sign(g_m[i]) with probability |g_m[i]| / norm_m, else 0          (ssv_qsgd_quantize)
 *     a[i]      = (1/M) sum_m norm_m q_m[i] ;  x[i] <- x[i] - lr a[i]              (ssv_qsgd_aggregate_apply)
 *
 * Conventions of this library (the paper fixes none of them):
 *   - the random choice is driven by an INPUT array of uniform numbers u in [0, 1), one per worker-coordinate:
 *     coordinate i is kept  <=>  u[i] * norm < |g[i]|, evaluated in fp32 (product rounded once).  A zero or NaN
 *     component is never kept; with norm 0 nothing is kept.
 *   - the norm is accumulated in double precision and rounded once to fp32; NaN does not take part in the maximum.
 *   - message format: two bit planes per worker, "nonzero" and "sign" (sign bit 1 <-> +1; 0 wherever the nonzero
 *     bit is 0), packed as in signvote.h (coordinate 64 w + i is bit i of word w, padding bits written 0 and
 *     ignored on input): the 2 d bits that always hold d numbers in {0, +-1}.
 *   - 1-way aggregate: a[i] = (sum over m = 0 .. M-1 in that order of +-norm_m or 0, in fp32) * (1/M), 1/M rounded
 *     once to fp32; update x <- fma(-lr, a, x); bf16 weights are widened, updated, rounded to nearest even.
 *
 * Pointers are DEVICE memory owned by the caller; layouts, streams, alignment rules and status codes are those of
 * signvote.h.  Nothing is allocated: ssv_qsgd_norms takes its scratch space (per-workgroup partial sums) from the
 * caller as `workspace`.
 */
#ifndef SIGNVOTE_QSGD_H
#define SIGNVOTE_QSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSV_QSGD_L2 0
#define SSV_QSGD_MAX 1

/* Bytes of workspace ssv_qsgd_norms needs for M rows (it does not depend on d); 0 if M is out of range. */
size_t ssv_qsgd_workspace_bytes(int M);

/*
 * norms[m] = ||g[m]||_2 (kind = SSV_QSGD_L2) or max_i |g[m][i]| (SSV_QSGD_MAX) for the M rows of g
 * (Appendix B: the scale each quantiser divides by).
 *   g          device, M rows of d elements of type g_dt, row stride g_row_stride elements
 *   norms      device, M floats (output)
 *   workspace  device, at least ssv_qsgd_workspace_bytes(M) bytes, 8-byte aligned; contents on entry are
 *              irrelevant and are overwritten.  Two calls that overlap in time must not share it.
 */
int ssv_qsgd_norms(const void* g, int g_dt, int M, int64_t d, int64_t g_row_stride, int kind, float* norms,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * ssv_qsgd_norms for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and errors as
 * ssv_qsgd_norms, but the partial results live in a fixed array inside the library (512 KiB per GPU, held until
 * the process ends) instead of `workspace`; the call allocates and frees nothing.
 *   Limit: M <= 256 rows, else SSV_ERR_SHAPE.
 *   All calls on one GPU share that array: calls that overlap in time on one GPU (different streams or threads)
 *   race and give wrong norms; calls on one stream, or otherwise ordered, are safe.
 *   The array's device address is looked up on the first call on each GPU (SSV_ERR_HIP if that fails).
 */
int ssv_qsgd_norms_static(const void* g, int g_dt, int M, int64_t d, int64_t g_row_stride, int kind, float* norms,
                          void* stream);

/*
 * The ternary quantiser of Appendix B for every row: nonzero[m] / sign[m] bit i <- whether g[m][i] is kept / kept
 * and positive, with u[m][i] * norms[m] < |g[m][i]| as the keep rule.
 *   u          device, M rows of d fp32 uniforms in [0, 1), row stride u_row_stride
 *   norms      device, M floats (from ssv_qsgd_norms, or any scale the caller chooses)
 *   nonzero, sign   device, M packed rows each, row stride row_stride_words (>= ceil(d/64))
 */
int ssv_qsgd_quantize(const void* g, int g_dt, const float* u, const float* norms, int M, int64_t d,
                      int64_t g_row_stride, int64_t u_row_stride, uint64_t* nonzero, uint64_t* sign,
                      int64_t row_stride_words, void* stream);

/*
 * Server side of the 1-way scheme (the QSGD figure of Section 4: the aggregate is not compressed again) fused with
 * the SGD update: a = average over the M workers of norms[m] * q_m, x <- x - lr a.
 *   avg_out    optional, device, d floats: receives a
 *   x          optional, device, d elements of x_dt, updated in place
 * At least one of avg_out and x must be given.
 */
int ssv_qsgd_aggregate_apply(const uint64_t* nonzero, const uint64_t* sign, const float* norms, int M, int64_t d,
                             int64_t row_stride_words, float* avg_out, void* x, int x_dt, float lr, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SIGNVOTE_QSGD_H */
