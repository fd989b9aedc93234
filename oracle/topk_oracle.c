/*
 * CPU oracle for top-k selection.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the parity reference for the GPU library: a plain, slow,
 * single-threaded program that writes out the textbook definition of the
 * operation.  It shares no code, header, table or helper with the GPU path and
 * must never be linked into or called from it.  Only the test-suite, the smoke
 * check and the benchmark's "cpu_baseline" leg use it.
 *
 * What it computes (paper, Section 1, problem statement: the k largest or
 * smallest of n elements, returned with their positions in the input;
 * Section 2.3.1: the pivot is the k-th element and the output is every element
 * on the better side of it, exactly k of them):
 *
 *   1. A total preorder "rank" on elements, written with floating-point
 *      comparisons on the decoded value (never with integer tricks on the bit
 *      pattern):  every NaN is greater than every non-NaN and all NaNs are
 *      equal to one another;  otherwise numeric order;  numerically equal
 *      values (only +0 and -0) are ordered by sign, -0 below +0.
 *   2. All (element, index) pairs of a row are sorted:  for "largest", a comes
 *      before b iff rank(a) > rank(b), or the ranks are equal and a's index is
 *      lower;  for "smallest", iff rank(a) < rank(b), or equal and a's index
 *      is lower.
 *   3. The first k pairs are the answer, in that order.  values[j] carries the
 *      element's original bit pattern, indices[j] its position in the row.
 *
 * The paper does not say how floats map to radix keys, how signed zeros, NaN
 * or ties at the k-th element are treated; the rules above are this build's
 * reading (IEEE totalOrder on non-NaN values, one NaN class on top, lowest
 * index first among equals).
 *
 * A second, independent selector (repeated arg-best scan, O(n*k)) is provided
 * so that the sort-based oracle can be pinned against brute force on small
 * inputs.
 *
 * Precision: 16-bit inputs are decoded exactly to double; fp32 is widened to
 * double exactly.  No arithmetic is performed on values, only comparisons.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

/* ---- decoding of storage formats to double (exact) ---------------------- */

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0x1f) {
        v = f ? NAN : INFINITY;
    } else if (e == 0) {
        v = ldexp((double)f, -24);            /* subnormal: f * 2^-10 * 2^-14 */
    } else {
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    }
    return sign ? -v : v;
}

/* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
static double decode_bf16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xff;
    int f = h & 0x7f;
    double v;
    if (e == 0xff) {
        v = f ? NAN : INFINITY;
    } else if (e == 0) {
        v = ldexp((double)f, -133);           /* f * 2^-7 * 2^-126 */
    } else {
        v = ldexp(1.0 + (double)f / 128.0, e - 127);
    }
    return sign ? -v : v;
}

static int elem_size(int dtype)
{
    return dtype == ORACLE_F32 ? 4 : 2;
}

/* Decoded value of element i of a row, plus its raw bits (zero-extended). */
static double decode_at(const void *row, int dtype, int64_t i, uint32_t *bits)
{
    if (dtype == ORACLE_F32) {
        uint32_t b;
        float f;
        memcpy(&b, (const char *)row + 4 * i, 4);
        memcpy(&f, &b, 4);
        *bits = b;
        return (double)f;
    } else {
        uint16_t h;
        memcpy(&h, (const char *)row + 2 * i, 2);
        *bits = h;
        return dtype == ORACLE_F16 ? decode_f16(h) : decode_bf16(h);
    }
}

/* Exported for the tests that pin the decoders against numpy / torch. */
double oracle_decode(int dtype, uint32_t bits)
{
    if (dtype == ORACLE_F32) {
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
    return dtype == ORACLE_F16 ? decode_f16((uint16_t)bits) : decode_bf16((uint16_t)bits);
}

/* ---- the preorder -------------------------------------------------------- */

typedef struct {
    double x;       /* decoded value (NaN allowed)     */
    int64_t idx;    /* position in the row             */
} item_t;

/* -1 if a ranks below b, 0 if equal rank, +1 if above. */
static int rank_cmp(double a, double b)
{
    int an = isnan(a), bn = isnan(b);
    if (an || bn) return an - bn;             /* NaN above everything, NaNs tie */
    if (a < b) return -1;
    if (a > b) return 1;
    /* numerically equal: only the two zeros differ */
    {
        int as = signbit(a) ? 1 : 0, bs = signbit(b) ? 1 : 0;
        return bs - as;                       /* -0 (sign 1) below +0 (sign 0) */
    }
}

/* Exported so tests can probe the preorder directly. */
int oracle_rank_cmp(int dtype, uint32_t abits, uint32_t bbits)
{
    return rank_cmp(oracle_decode(dtype, abits), oracle_decode(dtype, bbits));
}

static int cmp_largest(const void *pa, const void *pb)
{
    const item_t *a = (const item_t *)pa, *b = (const item_t *)pb;
    int r = rank_cmp(a->x, b->x);
    if (r > 0) return -1;                     /* higher rank first */
    if (r < 0) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

static int cmp_smallest(const void *pa, const void *pb)
{
    const item_t *a = (const item_t *)pa, *b = (const item_t *)pb;
    int r = rank_cmp(a->x, b->x);
    if (r < 0) return -1;                     /* lower rank first */
    if (r > 0) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/* ---- full ordering of one row ------------------------------------------- */

/*
 * order_out[j] = index of the j-th pair of the row in the oracle's order
 * (j = 0 is the best element).  Any k is then answered by the first k entries.
 * Returns 0 on success, 1 on bad arguments, 2 if memory ran out.
 */
int oracle_sort_row(const void *row, int dtype, int64_t n, int largest, int64_t *order_out)
{
    item_t *items;
    int64_t i;
    if (!row || !order_out || n < 1 || dtype < 0 || dtype > 2) return 1;
    items = (item_t *)malloc((size_t)n * sizeof(item_t));
    if (!items) return 2;
    for (i = 0; i < n; ++i) {
        uint32_t bits;
        items[i].x = decode_at(row, dtype, i, &bits);
        items[i].idx = i;
    }
    qsort(items, (size_t)n, sizeof(item_t), largest ? cmp_largest : cmp_smallest);
    for (i = 0; i < n; ++i) order_out[i] = items[i].idx;
    free(items);
    return 0;
}

/*
 * Top-k of every row of a [batch, n] row-major array by sorting the whole row.
 * out_values: [batch, k] in the input's storage format (original bits);
 * out_indices: [batch, k] int64 positions within the row.  Output rows are in
 * the oracle's order (best first, lowest index first among equals).
 */
int oracle_topk_sort(const void *keys, int dtype, int64_t batch, int64_t n, int64_t k,
                     int largest, void *out_values, int64_t *out_indices)
{
    int64_t *order;
    int64_t r, j;
    int es;
    if (!keys || !out_values || !out_indices) return 1;
    if (batch < 1 || n < 1 || k < 1 || k > n || dtype < 0 || dtype > 2) return 1;
    es = elem_size(dtype);
    order = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!order) return 2;
    for (r = 0; r < batch; ++r) {
        const char *row = (const char *)keys + (size_t)r * (size_t)n * es;
        int rc = oracle_sort_row(row, dtype, n, largest, order);
        if (rc) { free(order); return rc; }
        for (j = 0; j < k; ++j) {
            memcpy((char *)out_values + ((size_t)r * k + j) * es, row + (size_t)order[j] * es, es);
            out_indices[r * k + j] = order[j];
        }
    }
    free(order);
    return 0;
}

/*
 * Independent brute force: k rounds, each scanning the row for the best
 * not-yet-taken element (first one found wins ties, i.e. the lowest index).
 * O(n*k); for pinning the sort-based oracle on small inputs.
 */
int oracle_topk_bruteforce(const void *keys, int dtype, int64_t batch, int64_t n, int64_t k,
                           int largest, void *out_values, int64_t *out_indices)
{
    unsigned char *taken;
    int64_t r, j, i;
    int es;
    if (!keys || !out_values || !out_indices) return 1;
    if (batch < 1 || n < 1 || k < 1 || k > n || dtype < 0 || dtype > 2) return 1;
    es = elem_size(dtype);
    taken = (unsigned char *)malloc((size_t)n);
    if (!taken) return 2;
    for (r = 0; r < batch; ++r) {
        const char *row = (const char *)keys + (size_t)r * (size_t)n * es;
        memset(taken, 0, (size_t)n);
        for (j = 0; j < k; ++j) {
            int64_t best = -1;
            double bestx = 0.0;
            for (i = 0; i < n; ++i) {
                uint32_t bits;
                double x;
                int c;
                if (taken[i]) continue;
                x = decode_at(row, dtype, i, &bits);
                if (best < 0) { best = i; bestx = x; continue; }
                c = rank_cmp(x, bestx);
                if (largest ? (c > 0) : (c < 0)) { best = i; bestx = x; }
            }
            taken[best] = 1;
            memcpy((char *)out_values + ((size_t)r * k + j) * es, row + (size_t)best * es, es);
            out_indices[r * k + j] = best;
        }
    }
    free(taken);
    return 0;
}
