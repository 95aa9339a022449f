/*
 * CPU ORACLE for the generalized two-stage approximate Top-K.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.  It shares no code,
 * header, table or helper with the HIP library and must stay that way.
 *
 * What it computes is the definition of the method written out literally
 * (paper Section 6.1, Steps 1-4), with no blocking, fusion or early exit:
 *
 *   Step 1  bucket i of a row holds the elements whose position n satisfies
 *           n mod B == i  (0-based form of G_i = {a_{i+jB}}; Section 6.1 and
 *           the [batch, N/B, B] view of Section 6.3).
 *   Step 2  T_i = the K' greatest elements of bucket i.
 *   Step 3  S   = union of all T_i            (B*K' elements).
 *   Step 4  output = the K greatest elements of S, listed greatest first.
 *
 * "Greatest" needs a total order.  The paper leaves ties open (its listing is
 * explicitly unstable); this build fixes them: element a comes before element
 * b when value(a) > value(b), or the values compare equal and index(a) <
 * index(b).  Values are compared numerically (so -0.0 equals +0.0 and the
 * index decides); outputs carry the stored bits of the chosen element.
 * Precondition: no NaN in the input (checked, returns -2).
 *
 * bf16 and fp16 inputs are widened to binary32 before comparing (exact and
 * order preserving), 32-bit integers are compared as integers: the promotion
 * rule of Section 6.3's listing.
 *
 * The exact Top-K (the K greatest of all N elements in the same order) is the
 * B = 1, K' = K case of the definition and is also provided on its own, written
 * separately, so the two can be checked against each other.
 *
 * Rows are independent (the batch axis is the only parallel axis in the
 * paper); the row loop carries an OpenMP pragma and nothing else is tuned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    double value;  /* numeric value used for comparisons */
    int32_t index; /* position n inside the row */
} element_t;

/*
 * Element types.  Section 6.3's listing promotes floating inputs of at most 32
 * bits to binary32, signed integers to int32 and unsigned ones to uint32 before
 * comparing.  Every value of those three compute types is exactly a binary64
 * number, so one comparison in double stands for all of them.
 */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2, ORACLE_I32 = 3, ORACLE_U32 = 4 };

/* IEEE binary16 -> binary32, written out field by field (exact). */
static float half_to_float(uint16_t h)
{
    int sign = h >> 15, exponent = (h >> 10) & 31, fraction = h & 1023;
    double magnitude;
    if (exponent == 31)
        magnitude = fraction ? NAN : INFINITY;
    else if (exponent == 0)
        magnitude = ldexp((double)fraction, -24);            /* subnormal: fraction * 2^-24 */
    else
        magnitude = ldexp(1.0 + fraction / 1024.0, exponent - 15);
    return (float)(sign ? -magnitude : magnitude);
}

static double widen(const void *row, int dtype, int64_t n)
{
    switch (dtype) {
    case ORACLE_F32:
        return ((const float *)row)[n];
    case ORACLE_BF16: {
        uint32_t bits = (uint32_t)((const uint16_t *)row)[n] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return f;
    }
    case ORACLE_F16:
        return half_to_float(((const uint16_t *)row)[n]);
    case ORACLE_I32:
        return ((const int32_t *)row)[n];
    default:
        return ((const uint32_t *)row)[n];
    }
}

static int known_dtype(int dtype) { return dtype >= ORACLE_F32 && dtype <= ORACLE_U32; }

static size_t elem_size(int dtype) { return (dtype == ORACLE_BF16 || dtype == ORACLE_F16) ? 2 : 4; }

/* qsort comparator: negative when a is "greater" (comes first). */
static int greater_first(const void *pa, const void *pb)
{
    const element_t *a = (const element_t *)pa;
    const element_t *b = (const element_t *)pb;
    if (a->value > b->value) return -1;
    if (a->value < b->value) return 1;
    if (a->index < b->index) return -1;
    if (a->index > b->index) return 1;
    return 0;
}

/*
 * The mirrored problem, the K smallest ("min-K"): element a comes before element b when
 * value(a) < value(b), or the values compare equal and index(a) < index(b).  Everything else
 * in the definition stays as it is, with "greatest" read as "first in this order".
 */
static int smaller_first(const void *pa, const void *pb)
{
    const element_t *a = (const element_t *)pa;
    const element_t *b = (const element_t *)pb;
    if (a->value < b->value) return -1;
    if (a->value > b->value) return 1;
    if (a->index < b->index) return -1;
    if (a->index > b->index) return 1;
    return 0;
}

typedef int (*order_fn)(const void *, const void *);

static void store_output(const void *row, int dtype, const element_t *e,
                         void *out_vals, int32_t *out_idx, int64_t pos)
{
    /* the stored bits of the chosen element, not a re-encoding of its value */
    size_t es = elem_size(dtype);
    memcpy((char *)out_vals + (size_t)pos * es,
           (const char *)row + (size_t)e->index * es, es);
    out_idx[pos] = e->index;
}

/* rows run in parallel; a failure in any of them is recorded once */
static void set_status(int *status, int code)
{
#pragma omp critical(atk_oracle_status)
    { *status = code; }
}

int atk_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Returns 0, -1 on bad arguments, -2 when a NaN is found, -3 on allocation failure. */
static int check_args(const void *values, int dtype, int64_t rows, int64_t N,
                      int64_t row_stride, int64_t K, int64_t Kp, int64_t B)
{
    if (!values || !known_dtype(dtype)) return -1;
    if (rows < 0 || N <= 0 || row_stride < N || N > 2147483647LL) return -1;
    if (B < 1 || N % B != 0) return -1;
    if (Kp < 1 || Kp > K || Kp > N / B) return -1;
    if (K > B * Kp || K > N) return -1;
    return 0;
}

/*
 * Stage 1 alone (Steps 1-2): survivors in the paper's physical layout
 * [rows, K', B] (Section 6.3): plane k holds, for every bucket, its k-th
 * greatest element.  surv_vals has the input dtype, surv_idx is int32.
 */
static int stage1_in_order(order_fn first, const void *values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int64_t Kp, int64_t B,
                           void *surv_vals, int32_t *surv_idx)
{
    int rc = check_args(values, dtype, rows, N, row_stride, Kp, Kp, B);
    if (rc) return rc;
    int64_t per_bucket = N / B;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const char *row = (const char *)values + (size_t)r * row_stride * elem_size(dtype);
        element_t *bucket = (element_t *)malloc(sizeof(element_t) * (size_t)per_bucket);
        if (!bucket) { set_status(&status, -3); continue; }
        for (int64_t b = 0; b < B; ++b) {
            for (int64_t j = 0; j < per_bucket; ++j) {
                int64_t n = b + j * B;
                bucket[j].value = widen(row, dtype, n);
                bucket[j].index = (int32_t)n;
                if (isnan(bucket[j].value)) set_status(&status, -2);
            }
            qsort(bucket, (size_t)per_bucket, sizeof(element_t), first);
            for (int64_t k = 0; k < Kp; ++k) {
                int64_t pos = k * B + b;
                store_output(row, dtype, &bucket[k],
                             (char *)surv_vals + (size_t)r * B * Kp * elem_size(dtype),
                             surv_idx + r * B * Kp, pos);
            }
        }
        free(bucket);
    }
    return status;
}

int atk_oracle_stage1(const void *values, int dtype, int64_t rows, int64_t N,
                      int64_t row_stride, int64_t Kp, int64_t B,
                      void *surv_vals, int32_t *surv_idx)
{
    return stage1_in_order(greater_first, values, dtype, rows, N, row_stride, Kp, B, surv_vals, surv_idx);
}

/* Steps 1-4. out_vals: [rows, K] in the input dtype; out_idx: [rows, K] int32. */
static int approx_in_order(order_fn first, const void *values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int64_t K, int64_t Kp, int64_t B,
                           void *out_vals, int32_t *out_idx)
{
    int rc = check_args(values, dtype, rows, N, row_stride, K, Kp, B);
    if (rc) return rc;
    int64_t per_bucket = N / B;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const char *row = (const char *)values + (size_t)r * row_stride * elem_size(dtype);
        element_t *bucket = (element_t *)malloc(sizeof(element_t) * (size_t)per_bucket);
        element_t *selected = (element_t *)malloc(sizeof(element_t) * (size_t)(B * Kp));
        if (!bucket || !selected) { set_status(&status, -3); free(bucket); free(selected); continue; }
        int64_t n_selected = 0;
        for (int64_t b = 0; b < B; ++b) {
            /* Step 1: gather bucket b */
            for (int64_t j = 0; j < per_bucket; ++j) {
                int64_t n = b + j * B;
                bucket[j].value = widen(row, dtype, n);
                bucket[j].index = (int32_t)n;
                if (isnan(bucket[j].value)) set_status(&status, -2);
            }
            /* Step 2: its K' greatest (first in the order) */
            qsort(bucket, (size_t)per_bucket, sizeof(element_t), first);
            /* Step 3: union */
            for (int64_t k = 0; k < Kp; ++k) selected[n_selected++] = bucket[k];
        }
        /* Step 4: sort the union, keep the first K */
        qsort(selected, (size_t)n_selected, sizeof(element_t), first);
        for (int64_t k = 0; k < K; ++k)
            store_output(row, dtype, &selected[k],
                         (char *)out_vals + (size_t)r * K * elem_size(dtype),
                         out_idx + r * K, k);
        free(bucket);
        free(selected);
    }
    return status;
}

int atk_oracle_approx_topk(const void *values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int64_t K, int64_t Kp, int64_t B,
                           void *out_vals, int32_t *out_idx)
{
    return approx_in_order(greater_first, values, dtype, rows, N, row_stride, K, Kp, B, out_vals, out_idx);
}

/* The same four steps for the K smallest. */
int atk_oracle_approx_mink(const void *values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int64_t K, int64_t Kp, int64_t B,
                           void *out_vals, int32_t *out_idx)
{
    return approx_in_order(smaller_first, values, dtype, rows, N, row_stride, K, Kp, B, out_vals, out_idx);
}

int atk_oracle_stage1_min(const void *values, int dtype, int64_t rows, int64_t N,
                          int64_t row_stride, int64_t Kp, int64_t B,
                          void *surv_vals, int32_t *surv_idx)
{
    return stage1_in_order(smaller_first, values, dtype, rows, N, row_stride, Kp, B, surv_vals, surv_idx);
}

/* Exact Top-K: the K greatest (first in the order) of all N elements of each row, in order. */
static int exact_in_order(order_fn first, const void *values, int dtype, int64_t rows, int64_t N,
                          int64_t row_stride, int64_t K, void *out_vals, int32_t *out_idx)
{
    if (!values || !known_dtype(dtype)) return -1;
    if (rows < 0 || N <= 0 || row_stride < N || N > 2147483647LL) return -1;
    if (K < 1 || K > N) return -1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const char *row = (const char *)values + (size_t)r * row_stride * elem_size(dtype);
        element_t *all = (element_t *)malloc(sizeof(element_t) * (size_t)N);
        if (!all) { set_status(&status, -3); continue; }
        for (int64_t n = 0; n < N; ++n) {
            all[n].value = widen(row, dtype, n);
            all[n].index = (int32_t)n;
            if (isnan(all[n].value)) set_status(&status, -2);
        }
        qsort(all, (size_t)N, sizeof(element_t), first);
        for (int64_t k = 0; k < K; ++k)
            store_output(row, dtype, &all[k],
                         (char *)out_vals + (size_t)r * K * elem_size(dtype),
                         out_idx + r * K, k);
        free(all);
    }
    return status;
}

int atk_oracle_topk(const void *values, int dtype, int64_t rows, int64_t N,
                    int64_t row_stride, int64_t K, void *out_vals, int32_t *out_idx)
{
    return exact_in_order(greater_first, values, dtype, rows, N, row_stride, K, out_vals, out_idx);
}

/* Exact min-K: the K smallest of each row, smallest first. */
int atk_oracle_mink(const void *values, int dtype, int64_t rows, int64_t N,
                    int64_t row_stride, int64_t K, void *out_vals, int32_t *out_idx)
{
    return exact_in_order(smaller_first, values, dtype, rows, N, row_stride, K, out_vals, out_idx);
}

/*
 * Maximum inner-product search (Section 7.3; appendix "Matmul-fused
 * implementation"): the rows whose Top-K is wanted are never given, they are
 * the products of Q query vectors with N database vectors,
 *     score[r][n] = sum over d of queries[r][d] * database[n][d].
 * Inputs are bf16 or fp16 bit patterns, vectors contiguous ([Q, D] and [N, D]).
 * A product of two such numbers is exact in binary64 and a binary64 sum of D of
 * them carries a relative error near 1e-16, so the score kept here, that sum
 * rounded once to binary32, is the correctly rounded inner product.  (A
 * binary32 accumulator, which is what the paper's kernel and matrix hardware
 * use, differs from it by rounding that depends on the summation order.)
 */
/* scores: [Q, N] binary32.  dtype: ORACLE_BF16 or ORACLE_F16 (products of two binary16
 * numbers are exact in binary64 as well). */
int atk_oracle_mips_scores(const uint16_t *queries, const uint16_t *database, int dtype,
                           int64_t Q, int64_t N, int64_t D, float *scores)
{
    if (!queries || !database || !scores || Q < 0 || N <= 0 || D <= 0) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F16) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < Q; ++r) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t d = 0; d < D; ++d)
                acc += widen(queries, dtype, r * D + d) * widen(database, dtype, n * D + d);
            scores[r * N + n] = (float)acc;
        }
    }
    return 0;
}

/*
 * Steps 1-4 of Section 6.1 applied to every row of the score matrix.
 * out_vals: [Q, K] binary32 scores; out_idx: [Q, K] database positions.
 */
int atk_oracle_mips_approx_topk(const uint16_t *queries, const uint16_t *database, int dtype,
                                int64_t Q, int64_t N, int64_t D,
                                int64_t K, int64_t Kp, int64_t B,
                                float *out_vals, int32_t *out_idx)
{
    if (!queries || !database || Q < 0 || N <= 0 || D <= 0) return -1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < Q; ++r) {
        float *row = (float *)malloc(sizeof(float) * (size_t)N);
        if (!row) { set_status(&status, -3); continue; }
        int rc = atk_oracle_mips_scores(queries + r * D, database, dtype, 1, N, D, row);
        if (!rc)
            rc = atk_oracle_approx_topk(row, ORACLE_F32, 1, N, N, K, Kp, B,
                                        out_vals + r * K, out_idx + r * K);
        if (rc) set_status(&status, rc);
        free(row);
    }
    return status;
}
