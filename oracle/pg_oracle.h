/*
 * pg_oracle.h -- CPU reference ("oracle") for a kernel chain that is captured once and
 * replayed with fresh inputs.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product library includes, links or calls this
 * file; it shares no code, header, table or constant with the HIP path.  It is slow on
 * purpose: every kernel is evaluated elementwise in fp64 from operands held in their storage
 * dtype, and the result is rounded once (round-to-nearest-even) to the storage dtype.
 *
 * What it defines
 *   - chain semantics: the kernels of one iteration run in order; an operand is either an
 *     external input of this iteration, a fixed weight, or an internal buffer written by an
 *     earlier kernel (paper, Sec. 4 "Graph-Capture Layer": the two classes of kernel
 *     parameter; Sec. 3 "Parameter Indirection": a replay is valid iff every kernel reads
 *     this iteration's data).  Copies, placeholders, pointer tables and graphs change where
 *     operands come from, never the arithmetic, so the oracle for every replay mode is the
 *     same plain run of the chain.
 *   - the per-kernel arithmetic (the paper does not define kernels; these are the benchmark
 *     chain's six ops, each written as its textbook formula).
 *   - the selection rule (paper, Sec. 4.3 "Selective CUDA Graphs": keep the fastest of the
 *     available variants, independently per graph).
 *
 * Pins: closed forms, library routines in fp64 and a pure-Python brute force, all in
 * tests/test_oracle_*.py.  Outputs at the benchmark's full sizes have no published values:
 * parity unpinned there except through the pins on each op and on the chain rule.
 */
#ifndef PG_ORACLE_H
#define PG_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_ADD = 0, ORC_MUL = 1, ORC_GELU = 2, ORC_RMSNORM = 3, ORC_GEMV = 4, ORC_SCALE_BIAS_RELU = 5 };
enum { ORC_NONE = 0, ORC_EXT = 1, ORC_INT = 2, ORC_WEIGHT = 3 };
enum { ORC_MODE_EAGER = 0, ORC_MODE_GRAPH_COPY = 1, ORC_MODE_GRAPH_INDIRECT = 2 };

/* One kernel of the chain.  Operand roles per op:
 *   ADD, MUL         in0 = a (n elements), in1 = b (>= m elements, read as b[i mod m])
 *   GELU             in0 = a
 *   RMSNORM          in0 = x [rows, cols], in1 = g [cols]; n = cols
 *   GEMV             in0 = W [n, cols] row-major, in1 = h [rows, cols]; out [rows, n]
 *   SCALE_BIAS_RELU  in0 = x [n] viewed as [N, C, inner], in1 = s [C], in2 = b [C]
 */
typedef struct {
    int32_t op;
    int32_t dtype;
    int32_t out_index;      /* internal buffer written (always ORC_INT) */
    int32_t in_kind[3];
    int32_t in_index[3];
    int64_t n;
    int64_t m;
    int64_t rows;
    int64_t cols;
    int64_t inner;
    int64_t channels;
    double eps;
} orc_kernel;

/* scalar codecs */
uint16_t orc_bf16_from_f64(double x);
double orc_bf16_to_f64(uint16_t bits);
float orc_f32_from_f64(double x);

/* unrounded scalar formulas (fp64) */
double orc_gelu_f64(double a);

/* Single ops on raw buffers of the given dtype.  Return 0, or -1 on a bad argument. */
int orc_op_add(int dtype, void *out, const void *a, const void *b, int64_t n, int64_t m);
int orc_op_mul(int dtype, void *out, const void *a, const void *b, int64_t n, int64_t m);
int orc_op_gelu(int dtype, void *out, const void *a, int64_t n);
int orc_op_rmsnorm(int dtype, void *out, const void *x, const void *g, int64_t rows, int64_t cols, double eps);
int orc_op_gemv(int dtype, void *out, const void *W, const void *h, int64_t rows, int64_t n_out, int64_t cols);
int orc_op_scale_bias_relu(int dtype, void *out, const void *x, const void *s, const void *b,
                           int64_t n, int64_t channels, int64_t inner);

/* Run kernels [k_begin, k_end) of a chain on one iteration's inputs.  ext / weights / ints are
 * arrays of host pointers to buffers in the kernels' storage dtypes; ints are overwritten.
 * Returns 0, or -(k+1) if kernel k is malformed. */
int orc_chain_run(const orc_kernel *k, int32_t k_begin, int32_t k_end,
                  const void *const *ext, const void *const *weights, void *const *ints);

/* Selection: for each segment the available variant of least cost; cost is [n_seg][3] in the
 * order eager, graph-copy, graph-indirect; NaN or +inf marks a variant that does not exist.
 * Ties keep the earlier variant.  Returns 0, or -(s+1) if segment s has no variant.
 * Costs are durations: the rule is stated for finite costs >= 0.  A negative finite cost is outside
 * its domain -- this routine simply compares it like any other number, the product's pg_select
 * refuses such a table as malformed -- so the two are compared on non-negative tables only. */
int orc_select(const double *cost, int32_t n_seg, uint8_t *mode_out);

#ifdef __cplusplus
}
#endif
#endif
