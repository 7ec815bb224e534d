/*
 * signvote.h -- C ABI of libsignvote: the data-parallel hot path of signSGD / Signum with
 * majority vote (arXiv 1810.05291, Algorithm 1) on one AMD MI355X (gfx950).
 *
 * The M workers of Algorithm 1 are M rows of caller-owned device buffers on one GPU:
 *     on worker m :  v_m <- (1 - beta) g_m + beta v_m ;  transmit sign(v_m) as 1 bit/coordinate
 *     on server   :  V <- sum_m sign(v_m) ;  transmit sign(V)
 *     everywhere  :  x <- x - eta (sign(V) + lambda x)
 * All operations are element-wise over the d coordinates.
 *
 * Conventions (the paper does not fix them; they are this library's stated readings):
 *   - sign(0) = +1: the transmitted bit is (value >= 0) under IEEE comparison, so +0 and -0 give
 *     bit 1, NaN gives bit 0, +-Inf give 1 / 0.
 *   - vote ties (even M, V = 0) give +1: vote bit = [#(bits set) >= (M + 1) / 2].
 *   - packed format: uint64 words, coordinate 64 w + i is bit i of word w (bit 0 = least
 *     significant), bit 1 <-> +1, bit 0 <-> -1.  A row of d coordinates has ceil(d / 64) words.
 *     Producers write the padding bits of the last word as 0; consumers ignore them.
 *   - fp32 arithmetic order: v <- fma(beta, v, (1 - beta) * g), (1 - beta) rounded once to fp32;
 *     x <- x + (-eta | +eta) when lambda == 0, else t = fma(lambda, x, s), x <- fma(-eta, t, x).
 *     bf16 values are widened to fp32 (exact), results rounded to nearest even.
 *
 * Memory and ownership: every pointer is DEVICE memory owned by the caller unless the argument
 * is documented as host memory.  The library allocates nothing, never frees, and keeps no state
 * between calls apart from the built-in scratch array of ssv_qsgd_norms_static (signvote_qsgd.h) and one
 * measurement switch read from the environment on first use:
 *     SSV_TUNE_STEP_SERIAL=0   let the momentum forms of the gradient-side kernels (ssv_signum_step with v,
 *                              ssv_signum_momentum_pack) keep all row loads of a worker group in
 *                              flight instead of one load per wavefront at a time.  Results are
 *                              identical; on MI355X it is slower.  It exists so that the two
 *                              schedules can be profiled against each other; leave it unset.
 * Matrices are row-major, one row per worker, with the row stride given in
 * elements (or in 64-bit words for packed rows).  Inputs must not overlap outputs.  v and x are
 * updated in place.
 *
 * Execution: `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 * enqueue kernels and return; the caller synchronises.  Calls on one stream run in order.
 *
 * Errors: every function returns SSV_OK (0) or a negative ssv_status.  Argument errors are
 * detected before anything is launched and leave all buffers untouched.  Nothing is printed,
 * nothing aborts.
 *
 * Alignment: base pointers of fp32 / bf16 / packed buffers must be aligned to their element size
 * (4 / 2 / 8 bytes), else SSV_ERR_ALIGN.  The fast paths need 16-byte aligned bases and row
 * strides that are multiples of 16 bytes; other shapes take a narrower-load path with the same
 * results.  For full speed start every row on a 128-byte boundary (pad the row strides): a
 * wavefront's 1 KiB accesses then cover whole cache lines (5-8% faster on the Signum step).
 */
#ifndef SIGNVOTE_H
#define SIGNVOTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSV_MAX_WORKERS 1023            /* 1 <= M <= SSV_MAX_WORKERS */
#define SSV_MAX_COORDS (1LL << 40)      /* 1 <= d <= SSV_MAX_COORDS  */

typedef enum { SSV_F32 = 0, SSV_BF16 = 1 } ssv_dtype;

typedef enum {
    SSV_OK = 0,
    SSV_ERR_NULL = -1,   /* a required pointer is NULL */
    SSV_ERR_SHAPE = -2,  /* d < 1, d > SSV_MAX_COORDS, M < 1, M > SSV_MAX_WORKERS, row stride < row length */
    SSV_ERR_ALIGN = -3,  /* a base pointer is not aligned to its element size */
    SSV_ERR_DTYPE = -4,  /* dtype is not SSV_F32 / SSV_BF16 */
    SSV_ERR_PARAM = -5,  /* beta outside [0, 1), lr or weight_decay not finite, momentum asked without v */
    SSV_ERR_HIP = -6     /* the HIP runtime refused the launch */
} ssv_status;

/*
 * Sign compression (Algorithm 1, the worker's send line; Section 4, bit-packing of sign tensors).
 * For each of the M rows of x:  signs[m][w] bit i = (x[m][64 w + i] >= 0).
 *   x      device, M rows of d elements of type dt, row stride x_row_stride elements (>= d)
 *   signs  device, M rows of ceil(d/64) uint64 words, row stride signs_row_stride_words (>= ceil(d/64))
 */
int ssv_sign_pack(const void* x, int dt, int M, int64_t d, int64_t x_row_stride,
                  uint64_t* signs, int64_t signs_row_stride_words, void* stream);

/*
 * Worker side of Signum (Algorithm 1, the worker's momentum line, then its send line).
 * v[m] <- (1 - beta) g[m] + beta v[m] in place (fp32), signs[m] = packed (v[m] >= 0).
 *   g      device, M rows of d elements of type g_dt, row stride g_row_stride
 *   v      device, M rows of d fp32, row stride v_row_stride, read and written
 *   beta   in [0, 1)
 */
int ssv_signum_momentum_pack(const void* g, int g_dt, float* v, int M, int64_t d,
                             int64_t g_row_stride, int64_t v_row_stride, float beta,
                             uint64_t* signs, int64_t signs_row_stride_words, void* stream);

/*
 * Server side (Algorithm 1, the server's two lines: sum the sign vectors, send back the sign of the sum):
 * vote[w] bit i = [ #{m : signs[m][w] bit i set} >= (M + 1) / 2 ], i.e. sign(sum_m +-1) with
 * ties to +1.  Padding bits of the inputs are ignored; those of `vote` are written 0.
 *   signs  device, M packed rows;  vote  device, ceil(d/64) words
 */
int ssv_majority_vote(const uint64_t* signs, int M, int64_t d, int64_t signs_row_stride_words,
                      uint64_t* vote, void* stream);

/*
 * Parameter update (Algorithm 1, the last line: every worker updates x): x <- x - lr (s + weight_decay x), s = +1
 * where the vote bit is set, else -1.  In place on x (d elements of type x_dt).
 */
int ssv_apply_sign_update(void* x, int x_dt, int64_t d, const uint64_t* vote,
                          float lr, float weight_decay, void* stream);

/*
 * Fused server + update: ssv_majority_vote followed by ssv_apply_sign_update in one kernel; the
 * vote never makes a round trip through memory.  vote_out may be NULL; when given it receives
 * the packed vote.
 */
int ssv_vote_apply(const uint64_t* signs, int M, int64_t d, int64_t signs_row_stride_words,
                   void* x, int x_dt, float lr, float weight_decay, uint64_t* vote_out,
                   void* stream);

/*
 * One whole iteration of Algorithm 1 for all M workers in one kernel: momentum, sign, vote and
 * update; signs and vote counts stay in registers.
 *   v == NULL    signSGD (the caption of Algorithm 1: beta = 0 turns Signum into signSGD): no momentum state is read or
 *                written and the sign is taken of g itself; beta must then be 0.
 *   v != NULL    Signum: v is updated in place as in ssv_signum_momentum_pack.
 *   vote_out     optional, ceil(d/64) words: the packed vote.
 *   signs_out    optional, M packed rows (stride signs_row_stride_words): what each worker
 *                transmitted (after worker_flip).  This buffer also selects the FASTEST form of
 *                the call: given it, the step runs as two kernels -- (momentum +) sign + pack one
 *                worker row after the other, then vote + update on the packed rows -- which for
 *                Signum on MI355X sustains 81% of the HBM peak against 75% for the single kernel
 *                that walks all M rows at once (71% at M = 31, 69% with unpadded rows, where the
 *                two-kernel form still reaches 80% and 77%).  Results are bit-identical.  Pass it
 *                whenever M * ceil(d/64) * 8 bytes can be spared.
 *   worker_flip  optional, HOST memory, M bytes: nonzero = that worker transmits the negation of
 *                its sign vector (the sign-inverting adversary of Definition 1 / Section 4.1).
 *                Its momentum stays honest.  Read before the call returns.
 */
int ssv_signum_step(const void* g, int g_dt, float* v, int M, int64_t d,
                    int64_t g_row_stride, int64_t v_row_stride, float beta,
                    void* x, int x_dt, float lr, float weight_decay,
                    uint64_t* vote_out, uint64_t* signs_out, int64_t signs_row_stride_words,
                    const uint8_t* worker_flip, void* stream);

/*
 * Multi-tensor form of ssv_signum_step (Section 4: fusing many small tensors into one operation saved
 * compression and communication cost).  A model's parameters are T separate tensors, and every worker's
 * gradient and momentum of a tensor may be an allocation of its own (where autograd left it).  One launch
 * runs Algorithm 1 over all of them: the index space is the concatenation of the tensors, each cut into
 * units of 4096 coordinates with its own ragged end, so no gradient is copied into a flat buffer.  The
 * result for every tensor equals ssv_signum_step on that tensor alone (without optional outputs).
 *
 * The tensors are described by a "plan", a block of bytes that holds only sizes, the device addresses given
 * here and byte offsets, so the same bytes serve on the host and on the device:
 *   1. size it:  bytes = ssv_multi_plan_bytes(T, M, n)            (0 = bad arguments)
 *   2. fill a HOST buffer of that size (8-byte aligned) with ssv_multi_plan_fill;
 *   3. copy the bytes to DEVICE memory (8-byte aligned) once; both copies stay owned by the caller and must
 *      stay unchanged while steps use them;
 *   4. every iteration: ssv_signum_step_multi(plan_host, plan_device, beta, lr, weight_decay, stream).
 *
 *   T        number of tensors (>= 1);  M workers;  n[t] >= 1 elements of tensor t, sum <= SSV_MAX_COORDS   (host array)
 *   x[t]     device address of tensor t's weights (x_dt)                                             (host array of T)
 *   g[t*M+m] device address of worker m's gradient of tensor t (g_dt, n[t] elements)                  (host array of T*M)
 *   v[t*M+m] device address of worker m's fp32 momentum of tensor t; v == NULL: signSGD, beta must be 0
 * Addresses must be aligned to their element size (else SSV_ERR_ALIGN); a tensor all of whose addresses are
 * 16-byte aligned (8-byte for bf16) takes the vector path, others a one-element-per-lane path with the same
 * results.  plan_fill touches no device memory; step_multi reads T, M and the layout from plan_host before
 * it returns, and its kernel reads the tables from plan_device.
 */
size_t ssv_multi_plan_bytes(int T, int M, const int64_t* n);
int ssv_multi_plan_fill(void* plan_host, size_t plan_bytes, int T, int M, const int64_t* n, void* const* x, int x_dt,
                        const void* const* g, int g_dt, float* const* v);
int ssv_signum_step_multi(const void* plan_host, const void* plan_device, float beta, float lr, float weight_decay,
                          void* stream);

/*
 * ssv_signum_step_multi in its faster, two-kernel form (Section 4, tensor fusion; Algorithm 1): momentum + sign +
 * pack one worker after the other with the packed signs written to `workspace`, then vote + update on the packed
 * rows -- the multi-tensor counterpart of giving `signs_out` to ssv_signum_step.  Same plan, same results.
 *   workspace        device memory owned by the caller, 16-byte aligned (128 recommended), at least
 *                    ssv_multi_workspace_bytes(plan_host) = M * 64 * (units of the plan) * 8 bytes, i.e. about
 *                    M * d / 8 bytes; contents on entry are irrelevant; on return it holds every worker's packed
 *                    signs (tensor t's words of worker m start at word m * stride + 64 * (units before t)).
 *                    Two calls that overlap in time must not share it.
 * ssv_multi_workspace_bytes returns 0 for a pointer that does not hold a filled plan.
 */
size_t ssv_multi_workspace_bytes(const void* plan_host);
int ssv_signum_step_multi_ws(const void* plan_host, const void* plan_device, void* workspace, size_t workspace_bytes,
                             float beta, float lr, float weight_decay, void* stream);

/* Static, NUL-terminated description of a status code (host memory, never freed). */
const char* ssv_status_string(int status);

/* Library version: major * 1000 + minor. */
int ssv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SIGNVOTE_H */
