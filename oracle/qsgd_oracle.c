/*
 * qsgd_oracle.c -- plain CPU oracle for the ternary ("1-bit") QSGD compressors that the paper compares
 * majority vote with (Appendix B, "Bits sent per iteration"; the QSGD figure of Section 4).
 *
 * TEST INFRASTRUCTURE ONLY, like signvote_oracle.c: nothing in the product path may call it, and it shares no
 * code with the HIP library.
 *
 * What Appendix B defines: 1-bit QSGD takes a gradient vector g and sets coordinate i to sign(g_i) with
 * probability |g_i| / ||g||, and to zero otherwise; "L2" QSGD uses the Euclidean norm, "max" QSGD the
 * largest magnitude.  The compressed vector stands for ||g|| * q with q in {-1, 0, +1}^d; in the 1-way scheme
 * the server averages the M decoded vectors and the average is used as the gradient without recompression.
 *
 * Readings where the text is silent (each stated where it is used):
 *   Q1  the random choice is driven by a uniform number u_i in [0, 1) that is an INPUT, one per coordinate:
 *       keep coordinate i  <=>  u_i * ||g|| < |g_i|, evaluated in fp32 (product rounded once, then compared),
 *       which happens with probability |g_i| / ||g||.  Consequences of IEEE arithmetic, not extra rules: a zero
 *       or NaN component is never kept; with ||g|| = 0 nothing is kept.
 *   Q2  the norm is computed in double precision (squares of fp32 numbers are exact in double), summed in index
 *       order, square-rooted and rounded once to fp32; NaN components do not take part in the maximum.
 *   Q3  message format: two bit planes of one bit per coordinate, "nonzero" and "sign" (sign bit 1 <-> +1, and 0
 *       wherever the nonzero bit is 0), packed like the sign vectors (coordinate 64 w + i <-> bit i of word w,
 *       padding bits 0): the 2 d bits that Appendix B says always suffice for d numbers in {0, +-1}.
 *   Q4  1-way aggregate: a_i = (sum over m = 0 .. M-1, in that order, of +-||g_m|| or 0, in fp32) * (1/M) with 1/M
 *       rounded once to fp32; update x_i <- fma(-eta, a_i, x_i); bf16 weights are widened, updated, and rounded
 *       to nearest even.
 *
 * Parity pins: tests/test_qsgd_oracle_pins.py.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORA_F32 0
#define ORA_BF16 1
#define ORA_QSGD_L2 0
#define ORA_QSGD_MAX 1

static float q_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t q_f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* ---------- the norm (Appendix B: ||g||_2 for L2 QSGD, ||g||_inf for max QSGD; reading Q2) ---------- */

double ora_qsgd_norm_f64(const float *g, int64_t d, int kind) {
    if (kind == ORA_QSGD_L2) {
        double acc = 0.0;
        for (int64_t i = 0; i < d; ++i) acc += (double)g[i] * (double)g[i];
        return sqrt(acc);
    }
    double mx = 0.0;
    for (int64_t i = 0; i < d; ++i) {
        double a = fabs((double)g[i]);
        if (a > mx) mx = a; /* false for NaN: it does not take part */
    }
    return mx;
}

/* ---------- the stochastic ternary choice (Appendix B; reading Q1) ---------- */

void ora_qsgd_quantize_row(const float *g, const float *u, int64_t d, float norm, int8_t *q) {
#pragma omp parallel for schedule(static) /* element-wise: order is immaterial */
    for (int64_t i = 0; i < d; ++i) {
        float threshold = u[i] * norm;
        int keep = threshold < fabsf(g[i]);
        q[i] = keep ? (g[i] > 0.0f ? 1 : -1) : 0;
    }
}

/* ---------- message format (reading Q3) ---------- */

void ora_qsgd_pack(const int8_t *q, int64_t d, uint64_t *nonzero, uint64_t *sign) {
    int64_t W = (d + 63) / 64;
    for (int64_t w = 0; w < W; ++w) {
        uint64_t nz = 0, sg = 0;
        for (int i = 0; i < 64; ++i) {
            int64_t j = 64 * w + i;
            if (j < d && q[j] != 0) nz |= (uint64_t)1 << i;
            if (j < d && q[j] > 0) sg |= (uint64_t)1 << i;
        }
        nonzero[w] = nz;
        sign[w] = sg;
    }
}

void ora_qsgd_unpack(const uint64_t *nonzero, const uint64_t *sign, int64_t d, int8_t *q) {
    for (int64_t j = 0; j < d; ++j) {
        int nz = (int)((nonzero[j / 64] >> (j % 64)) & 1u);
        int sg = (int)((sign[j / 64] >> (j % 64)) & 1u);
        q[j] = nz ? (sg ? 1 : -1) : 0;
    }
}

/* ---------- server, 1-way scheme: average of the decoded vectors (reading Q4) ---------- */

void ora_qsgd_average(const int8_t *q, const float *norms, int M, int64_t d, float *avg) {
    const float inv_m = 1.0f / (float)M;
#pragma omp parallel for schedule(static) /* over coordinates; the sum over workers stays in index order */
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int m = 0; m < M; ++m) {
            int8_t c = q[(int64_t)m * d + j];
            if (c > 0) acc += norms[m];
            if (c < 0) acc -= norms[m];
        }
        avg[j] = acc * inv_m;
    }
}

void ora_qsgd_average_f64(const int8_t *q, const float *norms, int M, int64_t d, double *avg) {
    for (int64_t j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int m = 0; m < M; ++m) acc += (double)q[(int64_t)m * d + j] * (double)norms[m];
        avg[j] = acc / (double)M;
    }
}

/* ---------- SGD update with the averaged decoded gradient ---------- */

void ora_qsgd_update_f32(float *x, const float *avg, int64_t d, float lr) {
    for (int64_t j = 0; j < d; ++j) x[j] = fmaf(-lr, avg[j], x[j]);
}

void ora_qsgd_update_bf16(uint16_t *x, const float *avg, int64_t d, float lr) {
    for (int64_t j = 0; j < d; ++j) x[j] = q_f32_to_bf16(fmaf(-lr, avg[j], q_bf16_to_f32(x[j])));
}

/* ====================================================================================
 * Composite entry points with the argument lists of the GPU library's C ABI, on host pointers.
 * ==================================================================================== */

static float *q_row_as_f32(const void *base, int dt, int64_t row, int64_t stride, int64_t d) {
    float *out = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    if (dt == ORA_F32) {
        memcpy(out, (const float *)base + row * stride, sizeof(float) * (size_t)d);
    } else {
        const uint16_t *h = (const uint16_t *)base + row * stride;
        for (int64_t i = 0; i < d; ++i) out[i] = q_bf16_to_f32(h[i]);
    }
    return out;
}

int ora_qsgd_norms(const void *g, int g_dt, int M, int64_t d, int64_t g_row_stride, int kind, float *norms) {
    if (!g || !norms || M < 1 || d < 1 || (kind != ORA_QSGD_L2 && kind != ORA_QSGD_MAX)) return -1;
    for (int m = 0; m < M; ++m) {
        float *gf = q_row_as_f32(g, g_dt, m, g_row_stride, d);
        norms[m] = (float)ora_qsgd_norm_f64(gf, d, kind);
        free(gf);
    }
    return 0;
}

int ora_qsgd_quantize(const void *g, int g_dt, const float *u, const float *norms, int M, int64_t d,
                      int64_t g_row_stride, int64_t u_row_stride, uint64_t *nonzero, uint64_t *sign,
                      int64_t row_stride_words) {
    if (!g || !u || !norms || !nonzero || !sign || M < 1 || d < 1) return -1;
    int8_t *q = (int8_t *)malloc((size_t)d);
    for (int m = 0; m < M; ++m) {
        float *gf = q_row_as_f32(g, g_dt, m, g_row_stride, d);
        ora_qsgd_quantize_row(gf, u + (int64_t)m * u_row_stride, d, norms[m], q);
        ora_qsgd_pack(q, d, nonzero + (int64_t)m * row_stride_words, sign + (int64_t)m * row_stride_words);
        free(gf);
    }
    free(q);
    return 0;
}

/* avg_out and x may each be NULL */
int ora_qsgd_aggregate_apply(const uint64_t *nonzero, const uint64_t *sign, const float *norms, int M, int64_t d,
                             int64_t row_stride_words, float *avg_out, void *x, int x_dt, float lr) {
    if (!nonzero || !sign || !norms || M < 1 || d < 1) return -1;
    int8_t *q = (int8_t *)malloc((size_t)M * (size_t)d);
    float *avg = (float *)malloc(sizeof(float) * (size_t)d);
    for (int m = 0; m < M; ++m)
        ora_qsgd_unpack(nonzero + (int64_t)m * row_stride_words, sign + (int64_t)m * row_stride_words, d,
                        q + (int64_t)m * d);
    ora_qsgd_average(q, norms, M, d, avg);
    if (avg_out) memcpy(avg_out, avg, sizeof(float) * (size_t)d);
    if (x) {
        if (x_dt == ORA_F32)
            ora_qsgd_update_f32((float *)x, avg, d, lr);
        else
            ora_qsgd_update_bf16((uint16_t *)x, avg, d, lr);
    }
    free(q);
    free(avg);
    return 0;
}
