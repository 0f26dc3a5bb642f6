/* Exercises every entry point of the CPU oracle on exactly-sized heap buffers with ragged shapes,
 * for a build with -fsanitize=address,undefined (tests/test_oracle_sanitizers.py): an access outside
 * an operand, a signed overflow or a misaligned load in the oracle ends the run with a report. */
#include "../oracle/pg_oracle.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static unsigned long long g_state = 0x9E3779B97F4A7C15ull;
static double unit(void)   /* a small deterministic generator: values in (-2, 2) */
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return ((double)(g_state >> 11) / 9007199254740992.0) * 4.0 - 2.0;
}

static void *make(int dtype, int64_t n)
{
    size_t eb = dtype == ORC_F32 ? 4 : 2;
    void *p = malloc((size_t)n * eb);   /* exactly n elements: one element too far is a heap overflow */
    if (!p) exit(3);
    for (int64_t i = 0; i < n; i++) {
        double v = unit();
        if (dtype == ORC_F32) ((float *)p)[i] = (float)v;
        else ((uint16_t *)p)[i] = orc_bf16_from_f64(v);
    }
    return p;
}

#define CHECK(x) do { if ((x) != 0) { fprintf(stderr, "failed: %s\n", #x); return 1; } } while (0)

int main(void)
{
    for (int dtype = 0; dtype < 2; dtype++) {
        /* elementwise, ragged n and a broadcast period that does not divide it */
        int64_t n = 1031, m = 7;
        void *a = make(dtype, n), *b = make(dtype, m), *bn = make(dtype, n), *o = make(dtype, n);
        CHECK(orc_op_add(dtype, o, a, b, n, m));
        CHECK(orc_op_mul(dtype, o, a, bn, n, n));
        CHECK(orc_op_gelu(dtype, o, a, n));
        CHECK(orc_op_add(dtype, a, a, b, n, 1));            /* in place, scalar operand */
        free(a); free(b); free(bn); free(o);
        /* rmsnorm and gemv, odd shapes */
        int64_t rows = 3, cols = 257, nout = 5;
        void *x = make(dtype, rows * cols), *g = make(dtype, cols), *y = make(dtype, rows * cols);
        CHECK(orc_op_rmsnorm(dtype, y, x, g, rows, cols, 1e-6));
        void *W = make(dtype, nout * cols), *z = make(dtype, rows * nout);
        CHECK(orc_op_gemv(dtype, z, W, x, rows, nout, cols));
        free(x); free(g); free(y); free(W); free(z);
        /* scale + bias + relu on [2, 3, 5] */
        void *t = make(dtype, 30), *s = make(dtype, 3), *bb = make(dtype, 3), *r = make(dtype, 30);
        CHECK(orc_op_scale_bias_relu(dtype, r, t, s, bb, 30, 3, 5));
        free(t); free(s); free(bb); free(r);
        /* a chain: x0 = e0 + e1; t = rmsnorm(x0 as [2,4]); y = W t; y = gelu(y); x0 = x0 * y */
        orc_kernel k[5];
        memset(k, 0, sizeof k);
        k[0].op = ORC_ADD; k[0].out_index = 0; k[0].in_kind[0] = ORC_EXT; k[0].in_index[0] = 0; k[0].in_kind[1] = ORC_EXT; k[0].in_index[1] = 1; k[0].n = 8; k[0].m = 8;
        k[1].op = ORC_RMSNORM; k[1].out_index = 1; k[1].in_kind[0] = ORC_INT; k[1].in_index[0] = 0; k[1].in_kind[1] = ORC_WEIGHT; k[1].in_index[1] = 0; k[1].n = 4; k[1].rows = 2; k[1].cols = 4; k[1].eps = 1e-3;
        k[2].op = ORC_GEMV; k[2].out_index = 2; k[2].in_kind[0] = ORC_WEIGHT; k[2].in_index[0] = 1; k[2].in_kind[1] = ORC_INT; k[2].in_index[1] = 1; k[2].n = 4; k[2].rows = 2; k[2].cols = 4;
        k[3].op = ORC_GELU; k[3].out_index = 2; k[3].in_kind[0] = ORC_INT; k[3].in_index[0] = 2; k[3].n = 8;
        k[4].op = ORC_MUL; k[4].out_index = 0; k[4].in_kind[0] = ORC_INT; k[4].in_index[0] = 0; k[4].in_kind[1] = ORC_INT; k[4].in_index[1] = 2; k[4].n = 8; k[4].m = 8;
        for (int i = 0; i < 5; i++) k[i].dtype = dtype;
        const void *ext[2] = {make(dtype, 8), make(dtype, 8)};
        const void *w[2] = {make(dtype, 4), make(dtype, 16)};
        void *ints[3] = {make(dtype, 8), make(dtype, 8), make(dtype, 8)};
        CHECK(orc_chain_run(k, 0, 5, ext, w, ints));
        CHECK(orc_chain_run(k, 2, 4, ext, w, ints));        /* a resumed stretch */
        for (int i = 0; i < 2; i++) { free((void *)ext[i]); free((void *)w[i]); }
        for (int i = 0; i < 3; i++) free(ints[i]);
    }
    /* codecs over every bf16 pattern, selection on a table with unavailable variants */
    for (uint32_t bits = 0; bits < 65536; bits++) (void)orc_bf16_from_f64(orc_bf16_to_f64((uint16_t)bits));
    (void)orc_bf16_from_f64(1e300); (void)orc_bf16_from_f64(-1e-300); (void)orc_f32_from_f64(1e-50);
    double nan = 0.0 / 0.0, inf = 1.0 / 0.0;
    double cost[9] = {3.0, 2.0, 2.0, 1.0, nan, inf, nan, 5.0, 4.0};
    uint8_t *mode = malloc(3);
    CHECK(orc_select(cost, 3, mode));
    if (mode[0] != 1 || mode[1] != 0 || mode[2] != 2) { fprintf(stderr, "selection wrong\n"); return 1; }
    free(mode);
    puts("oracle sanitizer driver: ok");
    return 0;
}
