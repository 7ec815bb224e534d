/*
 * signvote_oracle.c -- plain CPU oracle for Signum / signSGD with majority vote.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, by-eye-checkable statement of
 * what the method computes (Algorithm 1 of the paper, "Signum with majority
 * vote"); it exists so that the tests, the smoke check and the benchmark's
 * cpu_baseline leg have something independent to compare the GPU library with.
 * It shares no code, header, table or helper with the HIP library, and nothing
 * in the product path may call it.
 *
 * Every loop walks coordinates one at a time; signs are held as one int8 (+1/-1)
 * per coordinate and vote sums as plain int32 -- no bit tricks, no blocking, no
 * fusion.  The only parallelism is an OpenMP "parallel for" over coordinates,
 * which is legal because every operation of Algorithm 1 is element-wise.
 *
 * Readings of the paper that it is silent on (all stated where they are used):
 *   R1  sign(0) = +1  (the 1-bit message cannot carry a zero; test is  x >= 0,
 *       so +0, -0 -> +1; NaN -> -1 because the comparison is false; +-Inf -> +-1).
 *   R2  vote ties (even M, V = 0) -> +1, i.e. R1 applied to the sum V.
 *   R3  packed layout: 64 coordinates per uint64 word, coordinate 64w+i is bit i
 *       (LSB = bit 0) of word w, bit 1 <-> +1, padding bits of the last word 0.
 *   R4  storage precision: momentum v is fp32; gradients and weights fp32 or
 *       bf16.  The sign decision is taken on the fp32 value that is stored.
 *       fp32 arithmetic follows one fixed order:  v <- fma(beta, v, (1-beta)*g)
 *       with (1-beta) rounded once to fp32;  x <- x + (-/+ eta) when lambda = 0,
 *       else t = fma(lambda, x, s), x <- fma(-eta, t, x).  The *_f64 functions
 *       evaluate the same formulas in double for tolerance checks.
 *   R5  bf16 <- fp32 is round-to-nearest-even on the bit pattern; NaN keeps its
 *       sign and top payload bits and gets the quiet bit.
 *
 * Parity pins: tests/test_oracle_pins.py (brute force, closed forms, invariants,
 * the paper's worked example and binomial vote model).  No function here is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORA_F32 0
#define ORA_BF16 1

int ora_version(void) { return 1; }

int ora_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ora_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------- number formats (R5) ---------- */

static float bf16_bits_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16; /* bf16 is the top half of an fp32: exact */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t f32_to_bf16_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb; /* ties go to the even neighbour */
    return (uint16_t)(u >> 16);
}

void ora_bf16_to_f32(const uint16_t *h, int64_t n, float *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_bits_to_f32(h[i]);
}

void ora_f32_to_bf16(const float *x, int64_t n, uint16_t *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = f32_to_bf16_bits(x[i]);
}

/* ---------- sign (Algorithm 1, the worker's send line; reading R1) ---------- */

void ora_sign_f32(const float *x, int64_t n, int8_t *s) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) s[i] = (x[i] >= 0.0f) ? 1 : -1;
}

/* ---------- 1-bit message format (Section 4, bit-packing of sign tensors; R3) ---------- */

void ora_pack_signs(const int8_t *s, int64_t d, uint64_t *words) {
    int64_t W = (d + 63) / 64;
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < W; ++w) {
        uint64_t word = 0;
        for (int i = 0; i < 64; ++i) {
            int64_t j = 64 * w + i;
            if (j < d && s[j] > 0) word |= (uint64_t)1 << i;
        }
        words[w] = word;
    }
}

void ora_unpack_signs(const uint64_t *words, int64_t d, int8_t *s) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) s[j] = ((words[j / 64] >> (j % 64)) & 1u) ? 1 : -1;
}

/* ---------- momentum (Algorithm 1, the worker's momentum line) ---------- */

void ora_momentum_f32(const float *g, float *v, int64_t n, float beta) {
    const float omb = 1.0f - beta;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float t = omb * g[i];
        v[i] = fmaf(beta, v[i], t);
    }
}

void ora_momentum_f64(const float *g, const float *v, int64_t n, float beta, double *out) {
    const double b = (double)beta;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = (1.0 - b) * (double)g[i] + b * (double)v[i];
}

/* ---------- server: V = sum_m sign(v_m), then sign(V) (Algorithm 1; reading R2) ---------- */

void ora_vote_sum(const int8_t *s, int M, int64_t d, int64_t row_stride, int32_t *V) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        int32_t acc = 0;
        for (int m = 0; m < M; ++m) acc += s[(int64_t)m * row_stride + j];
        V[j] = acc;
    }
}

void ora_sign_i32(const int32_t *V, int64_t d, int8_t *s) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) s[j] = (V[j] >= 0) ? 1 : -1;
}

/* ---------- parameter update x <- x - eta (sign(V) + lambda x)  (Algorithm 1, last line) ---------- */

static float update_one_f32(float x, int8_t s, float lr, float wd) {
    if (wd == 0.0f) return x + (s > 0 ? -lr : lr);
    float t = fmaf(wd, x, (float)s);
    return fmaf(-lr, t, x);
}

void ora_apply_f32(float *x, int64_t d, const int8_t *vote, float lr, float wd) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) x[j] = update_one_f32(x[j], vote[j], lr, wd);
}

void ora_apply_bf16(uint16_t *x, int64_t d, const int8_t *vote, float lr, float wd) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j)
        x[j] = f32_to_bf16_bits(update_one_f32(bf16_bits_to_f32(x[j]), vote[j], lr, wd));
}

/* same formula in double from the stored inputs (x given as fp32 values) */
void ora_apply_f64(const float *x, int64_t d, const int8_t *vote, float lr, float wd, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j)
        out[j] = (double)x[j] - (double)lr * ((double)vote[j] + (double)wd * (double)x[j]);
}

/* ====================================================================================
 * Composite entry points: the same argument lists as the GPU library's C ABI, but on
 * host pointers.  Each one is the paper's steps called in the paper's order on whole
 * vectors, with unpacked int8 signs in between.  Return 0, or -1 for a bad argument.
 * ==================================================================================== */

static float *row_as_f32(const void *base, int dt, int64_t row, int64_t stride, int64_t d) {
    float *out = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    if (dt == ORA_F32)
        memcpy(out, (const float *)base + row * stride, sizeof(float) * (size_t)d);
    else
        ora_bf16_to_f32((const uint16_t *)base + row * stride, d, out);
    return out;
}

int ora_sign_pack(const void *x, int dt, int M, int64_t d, int64_t x_row_stride, uint64_t *signs,
                  int64_t signs_row_stride_words) {
    if (!x || !signs || M < 1 || d < 1 || (dt != ORA_F32 && dt != ORA_BF16)) return -1;
    int8_t *s = (int8_t *)malloc((size_t)d);
    for (int m = 0; m < M; ++m) {
        float *xf = row_as_f32(x, dt, m, x_row_stride, d);
        ora_sign_f32(xf, d, s);
        ora_pack_signs(s, d, signs + (int64_t)m * signs_row_stride_words);
        free(xf);
    }
    free(s);
    return 0;
}

int ora_signum_momentum_pack(const void *g, int g_dt, float *v, int M, int64_t d, int64_t g_row_stride,
                             int64_t v_row_stride, float beta, uint64_t *signs,
                             int64_t signs_row_stride_words) {
    if (!g || !v || !signs || M < 1 || d < 1) return -1;
    int8_t *s = (int8_t *)malloc((size_t)d);
    for (int m = 0; m < M; ++m) {
        float *gf = row_as_f32(g, g_dt, m, g_row_stride, d);
        float *vm = v + (int64_t)m * v_row_stride;
        ora_momentum_f32(gf, vm, d, beta);
        ora_sign_f32(vm, d, s);
        ora_pack_signs(s, d, signs + (int64_t)m * signs_row_stride_words);
        free(gf);
    }
    free(s);
    return 0;
}

/* vote on packed rows: unpack every row to +-1, add them up as integers, take the sign, pack. */
int ora_majority_vote(const uint64_t *signs, int M, int64_t d, int64_t signs_row_stride_words,
                      uint64_t *vote) {
    if (!signs || !vote || M < 1 || d < 1) return -1;
    int8_t *s = (int8_t *)malloc((size_t)M * (size_t)d);
    int32_t *V = (int32_t *)malloc(sizeof(int32_t) * (size_t)d);
    int8_t *sv = (int8_t *)malloc((size_t)d);
    for (int m = 0; m < M; ++m)
        ora_unpack_signs(signs + (int64_t)m * signs_row_stride_words, d, s + (int64_t)m * d);
    ora_vote_sum(s, M, d, d, V);
    ora_sign_i32(V, d, sv);
    ora_pack_signs(sv, d, vote);
    free(s);
    free(V);
    free(sv);
    return 0;
}

int ora_apply_sign_update(void *x, int x_dt, int64_t d, const uint64_t *vote, float lr, float wd) {
    if (!x || !vote || d < 1) return -1;
    int8_t *sv = (int8_t *)malloc((size_t)d);
    ora_unpack_signs(vote, d, sv);
    if (x_dt == ORA_F32)
        ora_apply_f32((float *)x, d, sv, lr, wd);
    else
        ora_apply_bf16((uint16_t *)x, d, sv, lr, wd);
    free(sv);
    return 0;
}

int ora_vote_apply(const uint64_t *signs, int M, int64_t d, int64_t signs_row_stride_words, void *x,
                   int x_dt, float lr, float wd, uint64_t *vote_out) {
    if (!signs || !x || M < 1 || d < 1) return -1;
    uint64_t *vote = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)((d + 63) / 64));
    ora_majority_vote(signs, M, d, signs_row_stride_words, vote);
    ora_apply_sign_update(x, x_dt, d, vote, lr, wd);
    if (vote_out) memcpy(vote_out, vote, sizeof(uint64_t) * (size_t)((d + 63) / 64));
    free(vote);
    return 0;
}

/*
 * One whole iteration of Algorithm 1 for all M workers.
 *   v == NULL (then beta must be 0)  ->  signSGD: no momentum state, the sign is taken of
 *                               the gradient itself (caption of Algorithm 1: beta = 0 gives signSGD).
 *                               With v given, the momentum line runs as written for any beta.
 *   worker_flip[m] != 0     ->  worker m transmits the negation of its sign vector
 *                               (the sign-inverting adversary of Definition 1 / Section 4.1);
 *                               its momentum stays honest.
 *   vote_out, signs_out may be NULL; signs_out holds what each worker transmitted.
 */
int ora_signum_step(const void *g, int g_dt, float *v, int M, int64_t d, int64_t g_row_stride,
                    int64_t v_row_stride, float beta, void *x, int x_dt, float lr, float wd,
                    uint64_t *vote_out, uint64_t *signs_out, int64_t signs_row_stride_words,
                    const uint8_t *worker_flip) {
    if (!g || !x || M < 1 || d < 1) return -1;
    if (v == NULL && beta != 0.0f) return -1;
    int8_t *s = (int8_t *)malloc((size_t)M * (size_t)d);
    int32_t *V = (int32_t *)malloc(sizeof(int32_t) * (size_t)d);
    int8_t *sv = (int8_t *)malloc((size_t)d);
    /* on the m-th worker */
    for (int m = 0; m < M; ++m) {
        float *gf = row_as_f32(g, g_dt, m, g_row_stride, d);
        int8_t *sm = s + (int64_t)m * d;
        if (v != NULL) {
            float *vm = v + (int64_t)m * v_row_stride;
            ora_momentum_f32(gf, vm, d, beta);
            ora_sign_f32(vm, d, sm);
        } else {
            ora_sign_f32(gf, d, sm);
        }
        if (worker_flip && worker_flip[m])
            for (int64_t j = 0; j < d; ++j) sm[j] = (int8_t)(-sm[j]);
        if (signs_out) ora_pack_signs(sm, d, signs_out + (int64_t)m * signs_row_stride_words);
        free(gf);
    }
    /* on the server */
    ora_vote_sum(s, M, d, d, V);
    ora_sign_i32(V, d, sv);
    if (vote_out) ora_pack_signs(sv, d, vote_out);
    /* on every worker */
    if (x_dt == ORA_F32)
        ora_apply_f32((float *)x, d, sv, lr, wd);
    else
        ora_apply_bf16((uint16_t *)x, d, sv, lr, wd);
    free(s);
    free(V);
    free(sv);
    return 0;
}
