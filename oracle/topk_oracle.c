/*
 * CPU oracle for bucketed approximate top-k (arxiv 2412.04358).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition of what the
 * GPU library must compute.  It shares no code with the HIP path, and nothing in
 * the product path may call it.
 *
 * What is computed, per row of an m x n row-major matrix (Section 2, "Algorithm
 * design choices", Stage 1 / Stage 2, and Figure 2 left):
 *
 *   Stage 1  element i belongs to bucket i mod b (Appendix A.1, interleaved
 *            assignment, the one used throughout the paper's experiments) or to
 *            bucket floor(b*i/n) (Appendix A.1, contiguous assignment).  Each bucket
 *            is sorted and its k_b largest elements are kept; the b lists are
 *            concatenated in bucket order (b*k_b candidates).
 *   Stage 2  only when b*k_b > k: the k largest of the candidates are kept.
 *
 * Conventions the paper leaves open and this build fixes:
 *   - "larger" is the strict total order  (v_a > v_b) or (v_a == v_b and i_a < i_b):
 *     equal values are ranked by lower column index, at every stage; +0 == -0.
 *     Values are compared after exact widening to float (bf16 -> f32 is exact).
 *     Rows must be NaN-free.
 *   - output order: without Stage 2, slot j*k_b + t holds the t-th largest of
 *     bucket j; with Stage 2 the k survivors are listed largest first.
 *   - n need not be a multiple of b: bucket j simply holds the indices that the
 *     assignment formula sends there (interleaved: j, j+b, j+2b, ... below n, the
 *     short buckets of Figure 2, whose pad cell is never selected); every bucket
 *     then has floor(n/b) or ceil(n/b) elements, and k_b <= floor(n/b) keeps each
 *     one long enough.
 *   - out_vals carries the element's own bits (the sign of a zero survives).
 *
 * exact top-k (the comparison point, Section 1): sort the whole row by the same
 * order, keep the first k.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_INTERLEAVED = 0, ORC_CONTIGUOUS = 1 };
enum { ORC_OK = 0, ORC_BAD_ARG = -1, ORC_NO_MEM = -2 };

typedef struct {
    float v;       /* value widened to float, used for comparison only */
    int32_t i;     /* column index inside the row */
    uint32_t raw;  /* original bits (low 16 used for bf16) */
} item_t;

static float widen(const void *x, int64_t pos, int dtype, uint32_t *raw)
{
    uint32_t bits;
    if (dtype == ORC_F32) {
        bits = ((const uint32_t *)x)[pos];
        *raw = bits;
    } else {
        uint16_t h = ((const uint16_t *)x)[pos];
        *raw = h;
        bits = ((uint32_t)h) << 16;
    }
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static void put_val(void *out, int64_t pos, int dtype, uint32_t raw)
{
    if (dtype == ORC_F32)
        ((uint32_t *)out)[pos] = raw;
    else
        ((uint16_t *)out)[pos] = (uint16_t)raw;
}

/* qsort comparator: a sorts before b when a is "larger" in the selection order */
static int by_rank(const void *pa, const void *pb)
{
    const item_t *a = (const item_t *)pa, *b = (const item_t *)pb;
    if (a->v > b->v) return -1;
    if (a->v < b->v) return 1;
    if (a->i < b->i) return -1;
    if (a->i > b->i) return 1;
    return 0;
}

/* Appendix A.1: the bucket of element i */
static int64_t bucket_of(int64_t i, int64_t n, int64_t b, int assignment)
{
    if (assignment == ORC_CONTIGUOUS)
        return (b * i) / n;
    return i % b;
}

static int approx_row(const void *x, int64_t row, int64_t n, int64_t k, int64_t b, int64_t k_b,
                      int dtype, int assignment, void *out_vals, int32_t *out_idx,
                      void *cand_vals, int32_t *cand_idx)
{
    /* the row's elements grouped by bucket, each group in increasing index order:
       start[j] .. start[j+1] is bucket j */
    item_t *grouped = (item_t *)malloc((size_t)n * sizeof(item_t));
    int64_t *start = (int64_t *)calloc((size_t)b + 1, sizeof(int64_t));
    int64_t *fill = (int64_t *)malloc((size_t)b * sizeof(int64_t));
    item_t *cand = (item_t *)malloc((size_t)(b * k_b) * sizeof(item_t));
    if (!grouped || !start || !fill || !cand) {
        free(grouped); free(start); free(fill); free(cand);
        return ORC_NO_MEM;
    }
    for (int64_t i = 0; i < n; ++i)
        start[bucket_of(i, n, b, assignment) + 1] += 1;
    for (int64_t j = 0; j < b; ++j) {
        start[j + 1] += start[j];
        fill[j] = start[j];
    }
    for (int64_t i = 0; i < n; ++i) {
        item_t *e = &grouped[fill[bucket_of(i, n, b, assignment)]++];
        e->v = widen(x, row * n + i, dtype, &e->raw);
        e->i = (int32_t)i;
    }

    /* Stage 1 */
    for (int64_t j = 0; j < b; ++j) {
        item_t *bucket = grouped + start[j];
        qsort(bucket, (size_t)(start[j + 1] - start[j]), sizeof(item_t), by_rank);
        for (int64_t t = 0; t < k_b; ++t)
            cand[j * k_b + t] = bucket[t];
    }
    if (cand_vals && cand_idx) {
        for (int64_t c = 0; c < b * k_b; ++c) {
            put_val(cand_vals, row * b * k_b + c, dtype, cand[c].raw);
            cand_idx[row * b * k_b + c] = cand[c].i;
        }
    }
    /* Stage 2 */
    if (b * k_b > k)
        qsort(cand, (size_t)(b * k_b), sizeof(item_t), by_rank);
    for (int64_t s = 0; s < k; ++s) {
        put_val(out_vals, row * k + s, dtype, cand[s].raw);
        out_idx[row * k + s] = cand[s].i;
    }
    free(grouped);
    free(start);
    free(fill);
    free(cand);
    return ORC_OK;
}

static int exact_row(const void *x, int64_t row, int64_t n, int64_t k, int dtype,
                     void *out_vals, int32_t *out_idx)
{
    item_t *all = (item_t *)malloc((size_t)n * sizeof(item_t));
    if (!all) return ORC_NO_MEM;
    for (int64_t i = 0; i < n; ++i) {
        all[i].v = widen(x, row * n + i, dtype, &all[i].raw);
        all[i].i = (int32_t)i;
    }
    qsort(all, (size_t)n, sizeof(item_t), by_rank);
    for (int64_t s = 0; s < k; ++s) {
        put_val(out_vals, row * k + s, dtype, all[s].raw);
        out_idx[row * k + s] = all[s].i;
    }
    free(all);
    return ORC_OK;
}

/*
 * x: host, m x n row-major, dtype ORC_F32 (float) or ORC_BF16 (uint16 bit patterns).
 * out_vals: host, m x k of the same dtype; out_idx: host, m x k int32.
 * cand_vals / cand_idx: optional (may be NULL) m x (b*k_b) Stage-1 candidates.
 * threads: rows are independent and are split over this many OpenMP threads.
 * Constraints (Section 2): 1 <= b <= n, 1 <= k_b <= min(k, floor(n/b)), b*k_b >= k.
 */
int orc_approx_topk_assign(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b,
                           int dtype, int assignment, void *out_vals, int32_t *out_idx,
                           void *cand_vals, int32_t *cand_idx, int threads)
{
    if (assignment != ORC_INTERLEAVED && assignment != ORC_CONTIGUOUS) return ORC_BAD_ARG;
    if (!x || !out_vals || !out_idx) return ORC_BAD_ARG;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return ORC_BAD_ARG;
    if (m < 1 || n < 1 || n > INT32_MAX || k < 1 || k > n) return ORC_BAD_ARG;
    if (b < 1 || b > n || k_b < 1 || k_b > k || k_b > n / b || b * k_b < k) return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
    int status = ORC_OK;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int64_t r = 0; r < m; ++r) {
        int rc = approx_row(x, r, n, k, b, k_b, dtype, assignment, out_vals, out_idx, cand_vals, cand_idx);
        if (rc != ORC_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* the interleaved assignment, as in all of the paper's experiments */
int orc_approx_topk(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b,
                    int dtype, void *out_vals, int32_t *out_idx,
                    void *cand_vals, int32_t *cand_idx, int threads)
{
    return orc_approx_topk_assign(x, m, n, k, b, k_b, dtype, ORC_INTERLEAVED, out_vals, out_idx,
                                  cand_vals, cand_idx, threads);
}

int orc_exact_topk(const void *x, int64_t m, int64_t n, int64_t k, int dtype,
                   void *out_vals, int32_t *out_idx, int threads)
{
    if (!x || !out_vals || !out_idx) return ORC_BAD_ARG;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return ORC_BAD_ARG;
    if (m < 1 || n < 1 || n > INT32_MAX || k < 1 || k > n) return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
    int status = ORC_OK;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int64_t r = 0; r < m; ++r) {
        int rc = exact_row(x, r, n, k, dtype, out_vals, out_idx);
        if (rc != ORC_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}
