/*
 * pg_oracle.c -- CPU reference for the replayed kernel chain.  TEST INFRASTRUCTURE ONLY; see
 * pg_oracle.h for what it defines, what pins it, and who may call it.
 *
 * Rule for every op: read operands in their storage dtype, widen to fp64 (exact), evaluate the
 * real-number formula in fp64, round once to the storage dtype with ties to even, store.
 * OpenMP is used only across independent outputs; every sum runs in index order, so results
 * do not depend on the thread count.
 */
#include "pg_oracle.h"

#include <math.h>
#include <string.h>

/* ---------- scalar codecs ------------------------------------------------------------- */

/* bf16 is the upper half of an IEEE binary32: 1 sign, 8 exponent, 7 fraction bits. */
double orc_bf16_to_f64(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round an fp64 value straight to bf16 (no intermediate fp32 rounding): pick the bf16 quantum
 * at the value's binade, scale, round to the nearest integer with ties to even, scale back. */
uint16_t orc_bf16_from_f64(double x)
{
    uint32_t u;
    float f;
    if (isnan(x)) return 0x7FC0u;
    if (isinf(x)) return x > 0 ? 0x7F80u : 0xFF80u;
    if (x == 0.0) return signbit(x) ? 0x8000u : 0x0000u;
    {
        int e;
        double q, r;
        (void)frexp(x, &e);   /* |x| = f * 2^e, f in [0.5, 1)  =>  binade exponent is e-1 */
        e -= 1;
        if (e < -126) e = -126;          /* subnormal range shares the quantum of the lowest normal binade */
        q = ldexp(1.0, e - 7);           /* spacing of bf16 values in this binade */
        r = nearbyint(x / q) * q;        /* default rounding mode: nearest, ties to even */
        if (fabs(r) >= ldexp(1.0, 128)) return x > 0 ? 0x7F80u : 0xFF80u;
        f = (float)r;                    /* exact: r has at most 8 significant bits */
    }
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

float orc_f32_from_f64(double x)
{
    return (float)x;    /* C conversion rounds to nearest-even in the default mode */
}

/* ---------- typed load / store --------------------------------------------------------- */

static double ld(int dtype, const void *p, int64_t i)
{
    if (dtype == ORC_F32) return (double)((const float *)p)[i];
    return orc_bf16_to_f64(((const uint16_t *)p)[i]);
}

static void st(int dtype, void *p, int64_t i, double v)
{
    if (dtype == ORC_F32) ((float *)p)[i] = orc_f32_from_f64(v);
    else ((uint16_t *)p)[i] = orc_bf16_from_f64(v);
}

static int bad_dtype(int dtype) { return dtype != ORC_F32 && dtype != ORC_BF16; }

/* ---------- ops ------------------------------------------------------------------------ */

/* GELU(a) = a * Phi(a), Phi the standard normal CDF, written with erfc so that the left tail
 * keeps its relative accuracy: Phi(a) = erfc(-a / sqrt 2) / 2. */
double orc_gelu_f64(double a)
{
    return 0.5 * a * erfc(-a / sqrt(2.0));
}

int orc_op_add(int dtype, void *out, const void *a, const void *b, int64_t n, int64_t m)
{
    int64_t i;
    if (bad_dtype(dtype) || n < 0 || m <= 0 || !out || !a || !b) return -1;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; i++) st(dtype, out, i, ld(dtype, a, i) + ld(dtype, b, i % m));
    return 0;
}

int orc_op_mul(int dtype, void *out, const void *a, const void *b, int64_t n, int64_t m)
{
    int64_t i;
    if (bad_dtype(dtype) || n < 0 || m <= 0 || !out || !a || !b) return -1;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; i++) st(dtype, out, i, ld(dtype, a, i) * ld(dtype, b, i % m));
    return 0;
}

int orc_op_gelu(int dtype, void *out, const void *a, int64_t n)
{
    int64_t i;
    if (bad_dtype(dtype) || n < 0 || !out || !a) return -1;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; i++) st(dtype, out, i, orc_gelu_f64(ld(dtype, a, i)));
    return 0;
}

/* Per row: ms = mean of squares; out = x * (ms + eps)^(-1/2) * g. */
int orc_op_rmsnorm(int dtype, void *out, const void *x, const void *g, int64_t rows, int64_t cols, double eps)
{
    int64_t r;
    if (bad_dtype(dtype) || rows < 0 || cols <= 0 || !out || !x || !g) return -1;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; r++) {
        int64_t i;
        double ss = 0.0, scale;
        for (i = 0; i < cols; i++) {
            double v = ld(dtype, x, r * cols + i);
            ss += v * v;
        }
        scale = 1.0 / sqrt(ss / (double)cols + eps);
        for (i = 0; i < cols; i++)
            st(dtype, out, r * cols + i, ld(dtype, x, r * cols + i) * scale * ld(dtype, g, i));
    }
    return 0;
}

/* y[r, j] = sum_i W[j, i] * h[r, i]; W is [n_out, cols] row-major. */
int orc_op_gemv(int dtype, void *out, const void *W, const void *h, int64_t rows, int64_t n_out, int64_t cols)
{
    int64_t t;
    if (bad_dtype(dtype) || rows < 0 || n_out < 0 || cols <= 0 || !out || !W || !h) return -1;
#pragma omp parallel for schedule(static)
    for (t = 0; t < rows * n_out; t++) {
        int64_t r = t / n_out, j = t % n_out, i;
        double acc = 0.0;
        for (i = 0; i < cols; i++) acc += ld(dtype, W, j * cols + i) * ld(dtype, h, r * cols + i);
        st(dtype, out, r * n_out + j, acc);
    }
    return 0;
}

/* out[b, c, p] = max(0, x[b, c, p] * s[c] + b[c]) over a contiguous [N, C, inner] tensor. */
int orc_op_scale_bias_relu(int dtype, void *out, const void *x, const void *s, const void *b,
                           int64_t n, int64_t channels, int64_t inner)
{
    int64_t i;
    if (bad_dtype(dtype) || n < 0 || channels <= 0 || inner <= 0 || !out || !x || !s || !b) return -1;
    if (n % (channels * inner) != 0) return -1;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; i++) {
        int64_t c = (i / inner) % channels;
        double v = ld(dtype, x, i) * ld(dtype, s, c) + ld(dtype, b, c);
        st(dtype, out, i, v > 0.0 ? v : 0.0);
    }
    return 0;
}

/* ---------- chain ---------------------------------------------------------------------- */

static const void *operand(const orc_kernel *k, int j, const void *const *ext,
                           const void *const *weights, void *const *ints)
{
    switch (k->in_kind[j]) {
    case ORC_EXT: return ext[k->in_index[j]];
    case ORC_WEIGHT: return weights[k->in_index[j]];
    case ORC_INT: return ints[k->in_index[j]];
    default: return NULL;
    }
}

int orc_chain_run(const orc_kernel *ks, int32_t k_begin, int32_t k_end,
                  const void *const *ext, const void *const *weights, void *const *ints)
{
    int32_t i;
    for (i = k_begin; i < k_end; i++) {
        const orc_kernel *k = &ks[i];
        const void *a = operand(k, 0, ext, weights, ints);
        const void *b = operand(k, 1, ext, weights, ints);
        const void *c = operand(k, 2, ext, weights, ints);
        void *out = ints[k->out_index];
        int rc;
        switch (k->op) {
        case ORC_ADD: rc = orc_op_add(k->dtype, out, a, b, k->n, k->m); break;
        case ORC_MUL: rc = orc_op_mul(k->dtype, out, a, b, k->n, k->m); break;
        case ORC_GELU: rc = orc_op_gelu(k->dtype, out, a, k->n); break;
        case ORC_RMSNORM: rc = orc_op_rmsnorm(k->dtype, out, a, b, k->rows, k->cols, k->eps); break;
        case ORC_GEMV: rc = orc_op_gemv(k->dtype, out, a, b, k->rows, k->n, k->cols); break;
        case ORC_SCALE_BIAS_RELU:
            rc = orc_op_scale_bias_relu(k->dtype, out, a, b, c, k->n, k->channels, k->inner);
            break;
        default: rc = -1;
        }
        if (rc != 0) return -(i + 1);
    }
    return 0;
}

/* ---------- selection ------------------------------------------------------------------ */

int orc_select(const double *cost, int32_t n_seg, uint8_t *mode_out)
{
    int32_t s;
    for (s = 0; s < n_seg; s++) {
        int best = -1, m;
        for (m = 0; m < 3; m++) {
            double c = cost[3 * s + m];
            if (!isfinite(c)) continue;
            if (best < 0 || c < cost[3 * s + best]) best = m;
        }
        if (best < 0) return -(s + 1);
        mode_out[s] = (uint8_t)best;
    }
    return 0;
}
