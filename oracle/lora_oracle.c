/*
 * CPU oracle for the co-batched heterogeneous-rank LoRA delta.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this file.  It
 * shares no code, layout, table or constant with the HIP library: adapters arrive as separate
 * dense row-major arrays (never the packed pool), there is no segment table and no permutation.
 *
 * What it computes.  The paper gives the delta only in words: a frozen base layer plus a pair of
 * small low-rank matrices per adapted layer whose inner dimension is the adapter's rank
 * (Background, "Low-Rank Adaptation"), with requests of different adapters and ranks executed in
 * one batch (Background, "Kernel Optimizations"), where no request should have to do work sized
 * for another request's rank (Motivation, "Effect of Co-serving Adapters of Different Ranks").
 * Written out, for token t routed to adapter a = token_adapter[t] with rank r_a and scale s_a:
 *
 *     v[t, j] = sum_{k < in}  x[t, k] * A_a[k, j]                      j < r_a
 *     y[t, o] = y0[t, o] + s_a * sum_{j < r_a} v[t, j] * B_a[j, o]      o < out
 *
 * and y[t, :] = y0[t, :] when a < 0 (token without adapter).  The method reaches exactly this
 * definition (no approximation), so the oracle is the definition: fp64 arithmetic on the exact
 * values of the bf16 inputs, k and j ascending, nothing blocked, fused or reordered.  Tokens are
 * independent, so the only parallelism is an OpenMP loop over tokens.
 *
 * Every function here is pinned by the CPU tests against things other than itself: exact brute
 * force through a materialised delta matrix on dyadic inputs, the merged dense product
 * x (W + s A B) when all tokens share an adapter (the paper's remark that an adapter can be merged
 * into the base weights, Related Work "Parameter Efficient Fine-Tuning"), token-order invariance,
 * rank-r = two rank-r/2 halves, zero-B / no-adapter rows unchanged, and closed forms for unit
 * vectors.  No function is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_value(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* v[j] = sum_k x[k] * A[k][j], A row-major [in][r]; k ascending. */
static void shrink_row(const uint16_t *x, const uint16_t *A, int in, int r, double *v)
{
    for (int j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int k = 0; k < in; ++k)
            acc += bf16_value(x[k]) * bf16_value(A[(size_t)k * r + j]);
        v[j] = acc;
    }
}

/* y[o] = y0[o] + s * sum_j v[j] * B[j][o], B row-major [r][out]; j ascending. */
static void expand_row(const double *v, const uint16_t *B, int r, int out, double s,
                       const double *y0, double *y)
{
    for (int o = 0; o < out; ++o) {
        double acc = 0.0;
        for (int j = 0; j < r; ++j)
            acc += v[j] * bf16_value(B[(size_t)j * out + o]);
        y[o] = (y0 ? y0[o] : 0.0) + s * acc;
    }
}

static int check_common(int n_rows, int in, int out, int n_adapters, const int32_t *ranks)
{
    if (n_rows < 0 || in <= 0 || out <= 0 || n_adapters < 0) return 1;
    for (int a = 0; a < n_adapters; ++a)
        if (ranks[a] <= 0) return 1;
    return 0;
}

/*
 * Shrink only.  rows: which tokens to evaluate (NULL = tokens 0..n_rows-1).  x is the full
 * [T][in] bf16 array, indexed by token.  v_out is [n_rows][v_stride] fp64; entries j >= r_a and
 * rows without adapter are set to 0.
 */
int oracle_lora_shrink(int n_rows, const int32_t *rows, int in, const uint16_t *x,
                       const int32_t *token_adapter, int n_adapters, const int32_t *ranks,
                       const uint16_t *const *A, double *v_out, int v_stride)
{
    if (check_common(n_rows, in, 1, n_adapters, ranks)) return 1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n_rows; ++i) {
        int t = rows ? rows[i] : i;
        int a = token_adapter[t];
        double *v = v_out + (size_t)i * v_stride;
        for (int j = 0; j < v_stride; ++j) v[j] = 0.0;
        if (a < 0) continue;
        if (a >= n_adapters || ranks[a] > v_stride) { bad = 1; continue; }
        shrink_row(x + (size_t)t * in, A[a], in, ranks[a], v);
    }
    return bad;
}

/*
 * Expand only, from a given v (fp64, [n_rows][v_stride], row i belongs to token rows[i]).
 * y0 (fp64, [n_rows][out]) may be NULL for zero.  y is [n_rows][out] fp64.
 */
int oracle_lora_expand(int n_rows, const int32_t *rows, int out, const double *v, int v_stride,
                       const int32_t *token_adapter, int n_adapters, const int32_t *ranks,
                       const float *scales, const uint16_t *const *B, const double *y0, double *y)
{
    if (check_common(n_rows, 1, out, n_adapters, ranks)) return 1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n_rows; ++i) {
        int t = rows ? rows[i] : i;
        int a = token_adapter[t];
        double *yi = y + (size_t)i * out;
        const double *y0i = y0 ? y0 + (size_t)i * out : NULL;
        if (a < 0) {
            for (int o = 0; o < out; ++o) yi[o] = y0i ? y0i[o] : 0.0;
            continue;
        }
        if (a >= n_adapters || ranks[a] > v_stride) { bad = 1; continue; }
        expand_row(v + (size_t)i * v_stride, B[a], ranks[a], out, (double)scales[a], y0i, yi);
    }
    return bad;
}

/*
 * The whole delta for the selected tokens: the two formulas above, one token at a time.
 * y0 and y are [n_rows][out] fp64 (row i = token rows[i]); y0 may be NULL for zero.
 */
int oracle_lora_apply(int n_rows, const int32_t *rows, int in, int out, const uint16_t *x,
                      const int32_t *token_adapter, int n_adapters, const int32_t *ranks,
                      const float *scales, const uint16_t *const *A, const uint16_t *const *B,
                      const double *y0, double *y)
{
    if (check_common(n_rows, in, out, n_adapters, ranks)) return 1;
    int rmax = 1;
    for (int a = 0; a < n_adapters; ++a)
        if (ranks[a] > rmax) rmax = ranks[a];
    int bad = 0;
#pragma omp parallel
    {
        double *v = (double *)malloc((size_t)rmax * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_rows; ++i) {
            int t = rows ? rows[i] : i;
            int a = token_adapter[t];
            double *yi = y + (size_t)i * out;
            const double *y0i = y0 ? y0 + (size_t)i * out : NULL;
            if (a < 0) {
                for (int o = 0; o < out; ++o) yi[o] = y0i ? y0i[o] : 0.0;
                continue;
            }
            if (a >= n_adapters || !v) { bad = 1; continue; }
            shrink_row(x + (size_t)t * in, A[a], in, ranks[a], v);
            expand_row(v, B[a], ranks[a], out, (double)scales[a], y0i, yi);
        }
        free(v);
    }
    return bad;
}

/*
 * The adapted layer as a whole: base projection plus delta, per token,
 *
 *     y[t, o] = sum_{k < in} x[t, k] * W[k, o]  +  s_a * sum_{j < r_a} v[t, j] * B_a[j, o]
 *
 * with v as above and the second term absent for tokens without adapter: the frozen base layer and the
 * low-rank pair added to it (Background, "Low-Rank Adaptation"), which is what a serving system computes
 * for every adapted projection (Motivation, Fig. 3 measures Q, K, V, O).  W is bf16 bits, row-major
 * [in][out].  fp64 throughout, k ascending, then j ascending; nothing is rounded.  Pinned by a
 * hand-worked case with a 3 x 2 base matrix, by the merged dense product x (W + s A B), by W = 0
 * (which must give oracle_lora_apply's bits) and by numpy's x W on rows without adapter.
 */
int oracle_lora_linear(int n_rows, const int32_t *rows, int in, int out, const uint16_t *x, const uint16_t *W,
                       const int32_t *token_adapter, int n_adapters, const int32_t *ranks,
                       const float *scales, const uint16_t *const *A, const uint16_t *const *B, double *y)
{
    if (check_common(n_rows, in, out, n_adapters, ranks)) return 1;
    int rmax = 1;
    for (int a = 0; a < n_adapters; ++a)
        if (ranks[a] > rmax) rmax = ranks[a];
    int bad = 0;
#pragma omp parallel
    {
        double *v = (double *)malloc((size_t)rmax * sizeof(double));
        double *base = (double *)malloc((size_t)out * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_rows; ++i) {
            int t = rows ? rows[i] : i;
            int a = token_adapter[t];
            double *yi = y + (size_t)i * out;
            const uint16_t *xt = x + (size_t)t * in;
            if (!v || !base || a >= n_adapters) { bad = 1; continue; }
            for (int o = 0; o < out; ++o) {
                double acc = 0.0;
                for (int k = 0; k < in; ++k)
                    acc += bf16_value(xt[k]) * bf16_value(W[(size_t)k * out + o]);
                base[o] = acc;
            }
            if (a < 0) {
                for (int o = 0; o < out; ++o) yi[o] = base[o];
                continue;
            }
            shrink_row(xt, A[a], in, ranks[a], v);
            expand_row(v, B[a], ranks[a], out, (double)scales[a], base, yi);
        }
        free(v);
        free(base);
    }
    return bad;
}
