/*
 * elora_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the batched multi-adapter LoRA
 * linear layer computes, written directly from the paper:
 *
 *   - LoRA keeps W in R^{d x d} frozen and adds A in R^{r x d}, B in R^{d x r}
 *     with r << d (Sec. 2.1, "Low-Rank Adaptation").
 *   - Batch LoRA inference (Sec. 3.4, the displayed equation at its end):
 *       [y_0 .. y_n] = W x [x_0 .. x_n] + [B_0 A_0 x_0, .., B_n A_n x_n]
 *     i.e. the base product is shared by the whole batch and every request
 *     adds the product with ITS OWN adapter.
 *   - The baseline of Sec. 4.3 does the adapter part sample by sample; the
 *     grouped form ("u-batches": adapter id -> list of sample indices,
 *     gather, one product per adapter, scatter back) reaches the same result.
 *
 * The equation in the paper carries no scale factor; this build applies the
 * conventional LoRA factor s = alpha / r per adapter (or a per-row override),
 * so   y_t = W x_t + s * B_i (A_i x_t),   i = adapter of row t.
 *
 * Only tests/, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP path.
 * Everything is widened exactly to double before any arithmetic, all sums run
 * in index order, and nothing is blocked, fused or reordered beyond what the
 * definitions above state.  `#pragma omp parallel for` over rows only changes
 * which core computes a row, never the order of any sum.
 *
 * Memory layouts (row-major, the paper's operator orientation):
 *   x [T, K]   one request token per row
 *   W [N, K]   so that y_t[n] = sum_k W[n,k] x_t[k]
 *   A_i [r_i, K],  B_i [N, r_i]
 * dtype codes: 0 = IEEE fp32, 1 = bfloat16 stored as uint16 bit patterns.
 * Adapters kept in 8-bit blocks (the paper stores all adapters in the format its
 * settings call "Q8_0", Sec. 5 "Model"): A_i / B_i are then int8 codes in the same
 * row-major shapes, cut into blocks of 32 consecutive values in that order (a
 * block may run across rows), with one fp16 scale per block:
 *     value = fp16_scale[flat_index / 32] * code.
 * An adapter is in that format when a scale array is given for it.
 * wfmt codes:  0 = W has the dtype above,
 *              1 = W is 4-bit group-wise: byte b of row n holds code(k=2b) in
 *                  its low nibble and code(k=2b+1) in its high nibble,
 *                  w[n,k] = fp16_scale[n, k/32] * (code - 8)
 *                  (symmetric "Q4_0"-style block of 32 named in Sec. 5's
 *                  settings; the byte order is this build's own).
 *              2 = W is 8-bit group-wise (the "Q8_0" base of Sec. 5's setting
 *                  S1): int8 code per weight, row-major [N, K],
 *                  w[n,k] = fp16_scale[n, k/32] * code.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1
#define ORACLE_W_SAME 0
#define ORACLE_W_INT4_G32 1
#define ORACLE_W_INT8_G32 2

/* ---------- exact widening of stored values to double ---------- */

static double widen_bf16(uint16_t bits)
{
    /* bfloat16 is the top half of an fp32: append 16 zero bits. */
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen_fp16(uint16_t h)
{
    /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* subnormal: m * 2^-10 * 2^-14 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

static double widen(int dtype, const void *p, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[idx];
    return widen_bf16(((const uint16_t *)p)[idx]);
}

/* entry `idx` (flat, row-major) of an adapter matrix: in the dtype above, or scale * code for 8-bit blocks */
static double adapter_at(int dtype, const void *p, const uint16_t *block_scales, size_t idx)
{
    if (block_scales == NULL)
        return widen(dtype, p, idx);
    return widen_fp16(block_scales[idx / 32]) * (double)((const int8_t *)p)[idx];
}

static double weight_at(int dtype, int wfmt, const void *W, const uint16_t *w_scales,
                        int K, int n, int k)
{
    if (wfmt == ORACLE_W_SAME)
        return widen(dtype, W, (size_t)n * K + k);
    if (wfmt == ORACLE_W_INT8_G32)
        return widen_fp16(w_scales[(size_t)n * (K / 32) + k / 32]) * (double)((const int8_t *)W)[(size_t)n * K + k];
    const uint8_t *row = (const uint8_t *)W + (size_t)n * (K / 2);
    uint8_t byte = row[k / 2];
    int code = (k & 1) ? (byte >> 4) : (byte & 0x0f);
    double s = widen_fp16(w_scales[(size_t)n * (K / 32) + k / 32]);
    return s * (double)(code - 8);
}

/* ---------- routing (integer work, Sec. 3.4 / 4.3) ---------- */

/*
 * Expand a segment table to one adapter id per row.  Segment s covers rows
 * seg_offsets[s] <= t < seg_offsets[s+1]; the table must start at 0, end at T
 * and be non-decreasing (empty segments are allowed and cover nothing).
 * Returns 0, or -1 if the table is malformed.
 */
int elora_oracle_rows_from_segments(int T, int n_seg, const int32_t *seg_offsets,
                                    const int32_t *seg_adapter, int32_t *row_adapter)
{
    if (n_seg < 0 || T < 0)
        return -1;
    if (n_seg == 0)
        return T == 0 ? 0 : -1;
    if (seg_offsets[0] != 0 || seg_offsets[n_seg] != T)
        return -1;
    for (int s = 0; s < n_seg; ++s)
        if (seg_offsets[s + 1] < seg_offsets[s])
            return -1;
    for (int s = 0; s < n_seg; ++s)
        for (int t = seg_offsets[s]; t < seg_offsets[s + 1]; ++t)
            row_adapter[t] = seg_adapter[s];
    return 0;
}

/*
 * The u-batch map of Sec. 3.4 / 4.3: adapter id -> indices of the samples
 * that use it.  perm lists the rows grouped by adapter, rows of one adapter in
 * their original order (a stable counting sort); group_offsets[i]..[i+1] is
 * adapter i's slice of perm.  Rows with no adapter (id < 0) come last, after
 * group_offsets[P].  Returns the number of non-empty groups.
 */
int elora_oracle_ubatches(int T, int P, const int32_t *row_adapter, int32_t *perm,
                          int32_t *group_offsets)
{
    for (int i = 0; i <= P; ++i)
        group_offsets[i] = 0;
    for (int t = 0; t < T; ++t)
        if (row_adapter[t] >= 0 && row_adapter[t] < P)
            group_offsets[row_adapter[t] + 1] += 1;
    int distinct = 0;
    for (int i = 0; i < P; ++i) {
        if (group_offsets[i + 1] > 0)
            ++distinct;
        group_offsets[i + 1] += group_offsets[i];
    }
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(P + 1));
    for (int i = 0; i <= P; ++i)
        cursor[i] = group_offsets[i];
    for (int t = 0; t < T; ++t) {
        int a = row_adapter[t];
        int g = (a >= 0 && a < P) ? a : P;
        perm[cursor[g]++] = t;
    }
    free(cursor);
    return distinct;
}

/* ---------- the linear layer, per-sample form (Sec. 4.3 baseline) ---------- */

/*
 * y[ri, ci] for the selected rows/columns (rows == NULL: all T rows in order;
 * cols == NULL: all N columns in order), as doubles, row-major
 * [n_rows_sel, n_cols_sel].
 *
 *   ranks[i], adapter_scale[i], A[i], B[i]   describe pool entry i (A[i]/B[i]
 *       may be NULL for entries no row uses)
 *   A_scales, B_scales   NULL, or per entry NULL (A[i]/B[i] in `dtype`) or the fp16
 *       block scales of an entry kept as int8 codes
 *   row_adapter[t]  adapter of row t, or < 0 for "base model only"
 *   row_scale       NULL, or one factor per row that replaces adapter_scale
 *   n_threads       <= 0: library default; the value used is returned.
 * Returns the number of threads used (>= 1), or a negative value on a bad
 * argument (adapter id >= P, missing A/B).
 */
int elora_oracle_linear(int dtype, int wfmt, int T, int K, int N,
                        const void *x, const void *W, const uint16_t *w_scales,
                        int P, const int32_t *ranks, const double *adapter_scale,
                        const void *const *A, const void *const *B,
                        const uint16_t *const *A_scales, const uint16_t *const *B_scales,
                        const int32_t *row_adapter, const float *row_scale,
                        int n_rows_sel, const int32_t *rows,
                        int n_cols_sel, const int32_t *cols,
                        double *y, int n_threads)
{
    if (rows == NULL)
        n_rows_sel = T;
    if (cols == NULL)
        n_cols_sel = N;
    for (int t = 0; t < T; ++t) {
        int i = row_adapter[t];
        if (i >= P)
            return -2;
        if (i >= 0 && (A[i] == NULL || B[i] == NULL))
            return -3;
    }
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
    used = omp_get_max_threads();
#endif
    (void)n_threads;

#pragma omp parallel for schedule(dynamic, 1)
    for (int ri = 0; ri < n_rows_sel; ++ri) {
        int t = rows ? rows[ri] : ri;
        int i = row_adapter[t];
        double *xt = (double *)malloc(sizeof(double) * (size_t)K);
        for (int k = 0; k < K; ++k)
            xt[k] = widen(dtype, x, (size_t)t * K + k);

        /* shrink: v = A_i x_t  (r_i values) */
        int r = (i >= 0) ? ranks[i] : 0;
        double *v = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        for (int j = 0; j < r; ++j) {
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                s += adapter_at(dtype, A[i], A_scales ? A_scales[i] : NULL, (size_t)j * K + k) * xt[k];
            v[j] = s;
        }
        double scale = 0.0;
        if (i >= 0)
            scale = row_scale ? (double)row_scale[t] : adapter_scale[i];

        for (int ci = 0; ci < n_cols_sel; ++ci) {
            int n = cols ? cols[ci] : ci;
            /* base: (W x_t)[n] */
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += weight_at(dtype, wfmt, W, w_scales, K, n, k) * xt[k];
            /* expand + combine: + s * (B_i v)[n] */
            if (i >= 0) {
                double d = 0.0;
                for (int j = 0; j < r; ++j)
                    d += adapter_at(dtype, B[i], B_scales ? B_scales[i] : NULL, (size_t)n * r + j) * v[j];
                acc += scale * d;
            }
            y[(size_t)ri * n_cols_sel + ci] = acc;
        }
        free(v);
        free(xt);
    }
    return used;
}

/* ---------- the same layer, grouped form (Sec. 3.4 "u-batch") ---------- */

/*
 * Follows the order of Sec. 3.4: (1) base product for the whole batch,
 * (2) group rows by adapter, (3) per group: gather the rows, one A product and
 * one B product for the group, (4) scale, add to the base result and scatter
 * back to the rows' original positions.  Full output y [T, N] only.  Exists so
 * that tests can check "grouped == per-sample", the claim the paper's design
 * rests on.  Single-threaded.
 */
int elora_oracle_linear_grouped(int dtype, int wfmt, int T, int K, int N,
                                const void *x, const void *W, const uint16_t *w_scales,
                                int P, const int32_t *ranks, const double *adapter_scale,
                                const void *const *A, const void *const *B,
                                const uint16_t *const *A_scales, const uint16_t *const *B_scales,
                                const int32_t *row_adapter, const float *row_scale,
                                double *y)
{
    /* (1) base, whole batch */
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += weight_at(dtype, wfmt, W, w_scales, K, n, k) *
                       widen(dtype, x, (size_t)t * K + k);
            y[(size_t)t * N + n] = acc;
        }
    /* (2) adapter id -> sample indices */
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    int32_t *offs = (int32_t *)malloc(sizeof(int32_t) * (size_t)(P + 1));
    elora_oracle_ubatches(T, P, row_adapter, perm, offs);
    for (int i = 0; i < P; ++i) {
        int m = offs[i + 1] - offs[i];
        if (m == 0)
            continue;
        if (A[i] == NULL || B[i] == NULL) {
            free(perm);
            free(offs);
            return -3;
        }
        int r = ranks[i];
        /* (3) gather the u-batch, then V = Xg A_i^T and D = V B_i^T */
        double *xg = (double *)malloc(sizeof(double) * (size_t)m * K);
        double *vg = (double *)malloc(sizeof(double) * (size_t)m * (r > 0 ? r : 1));
        for (int g = 0; g < m; ++g)
            for (int k = 0; k < K; ++k)
                xg[(size_t)g * K + k] = widen(dtype, x, (size_t)perm[offs[i] + g] * K + k);
        for (int g = 0; g < m; ++g)
            for (int j = 0; j < r; ++j) {
                double s = 0.0;
                for (int k = 0; k < K; ++k)
                    s += adapter_at(dtype, A[i], A_scales ? A_scales[i] : NULL, (size_t)j * K + k) * xg[(size_t)g * K + k];
                vg[(size_t)g * r + j] = s;
            }
        /* (4) scale, combine, scatter to the original row */
        for (int g = 0; g < m; ++g) {
            int t = perm[offs[i] + g];
            double scale = row_scale ? (double)row_scale[t] : adapter_scale[i];
            for (int n = 0; n < N; ++n) {
                double d = 0.0;
                for (int j = 0; j < r; ++j)
                    d += adapter_at(dtype, B[i], B_scales ? B_scales[i] : NULL, (size_t)n * r + j) * vg[(size_t)g * r + j];
                y[(size_t)t * N + n] += scale * d;
            }
        }
        free(vg);
        free(xg);
    }
    free(perm);
    free(offs);
    return 1;
}

/* Exposed so tests can pin the two widenings against independent decoders. */
double elora_oracle_widen_bf16(uint16_t bits) { return widen_bf16(bits); }
double elora_oracle_widen_fp16(uint16_t bits) { return widen_fp16(bits); }
double elora_oracle_weight_at(int dtype, int wfmt, const void *W, const uint16_t *w_scales,
                              int K, int n, int k)
{
    return weight_at(dtype, wfmt, W, w_scales, K, n, k);
}
