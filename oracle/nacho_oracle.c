#define _POSIX_C_SOURCE 200809L
/*
 * CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, serial, obviously-correct implementation of what the hot path
 * computes, written from the paper.  It shares no code with the HIP library
 * and is never called by it; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load this file's shared object.
 *
 * Two kinds of result live here.
 *
 *  (1) Partition boundaries follow the paper's hierarchical search
 *      (Section 3.2, Algorithm 1 "FindPartition") step by step, with the
 *      concrete cost of Section 4.2.2 (the number of stored non-zeros of every
 *      coiterated operand inside the queried sub-space, scaled by the extent
 *      of a broadcast dimension) evaluated on level formats Dense and
 *      Compressed (Section 4.2.1).  No blocking, no range tracking, no
 *      k-ary probing: one binary search per level, one lower-bound search per
 *      operand per probe.
 *
 *  (2) Values and output indices are the plain definitions:
 *        SpMV   y_i  = sum_j A_ij x_j
 *        SpMM   C_ik = sum_j A_ij B_jk
 *        union add: the sorted union of the operands' stored coordinates, each
 *        with the sum (in operand order) of the operands that store it; this
 *        is the k-finger coiteration of Section 2.1 with "any operand matches"
 *        in place of "all operands match" (Section 2.2 gives the two-level
 *        loop nest for DCSR).
 *        intersection multiply: the sorted intersection of the operands'
 *        stored coordinates, each with the product (in operand order) of the
 *        k values; the k-finger loop of Section 2.1 as printed ("all operands
 *        match"), for sparse vectors and for the columns of every CSR row.
 *        Coordinate lists (COO: a non-unique compressed level over a Singleton
 *        level, Section 4.2.1) coiterate coordinate pairs in the same two loops.
 *
 * Precision: products and sums are accumulated wider than the GPU's working
 * type (long double for the fp64 kernels, double for the fp32 kernels) and the
 * sum of absolute terms is returned beside every value so that a test can use
 * the tolerance  |got - ref| <= tol * max(|ref|, sum|terms|).
 *
 * Readings of points the paper leaves open:
 *   - search domain of a level is [0, N_m] (the 3-vector listing of Section
 *     4.2.3 searches (0, N]); for an interior query the result is < N_m;
 *   - the first boundary is the origin and the last is the end of the space,
 *     by definition (the worked example of Section 2.1 draws [0,2) first);
 *   - on a flat stretch of the cost function the HIGHEST coordinate is taken
 *     (Algorithm 1 and the listing agree; it is then a stored coordinate);
 *   - query p of P is floor(p * Q_total / P);
 *   - lower-bound windows are half-open and return the window end when no
 *     entry qualifies;
 *   - a dense operand that is only located into (x of SpMV, B of SpMM) adds
 *     no cost; SpMM uses loop order i -> j -> k with the dense k innermost.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ORA_DENSE 0
#define ORA_COMPRESSED 1
/* The two levels of a coordinate-list (COO) matrix in the level-format vocabulary of
 * Section 4.2.1 (Dense, Compressed, Singleton):
 *   NONUNIQUE  a Compressed level whose sorted coordinates may repeat (one entry per
 *              stored non-zero; pos = {0, nnz} at the top);
 *   SINGLETON  exactly one coordinate per position of the level above: position p of
 *              the level above has the single child position p with coordinate crd[p]. */
#define ORA_NONUNIQUE 2
#define ORA_SINGLETON 3
#define ORA_MAXL 3
#define ORA_MAXK 16

typedef struct {
    int32_t kind;         /* ORA_DENSE / ORA_COMPRESSED                      */
    int64_t extent;       /* N_m                                             */
    const int32_t *pos;   /* compressed: segment bounds, one per parent + 1  */
    const int32_t *crd;   /* compressed: coordinates                         */
} ora_level;

typedef struct {
    int32_t nlevels;
    ora_level lvl[ORA_MAXL];
} ora_tensor;

/* ---- coordinate-tree navigation ---------------------------------------- */

/* First position at level m+1 among the children of level-m position p
 * (also valid for p == one-past-the-last position). */
static int64_t child_begin(const ora_tensor *T, int m, int64_t p)
{
    const ora_level *c = &T->lvl[m + 1];
    if (c->kind == ORA_SINGLETON) return p;
    return (c->kind == ORA_COMPRESSED || c->kind == ORA_NONUNIQUE) ? (int64_t)c->pos[p] : p * c->extent;
}

/* Number of innermost (leaf) positions that precede every leaf below level-m
 * position p, i.e. the leaf position where p's sub-tree starts. */
static int64_t leaf_begin(const ora_tensor *T, int m, int64_t p)
{
    for (; m + 1 < T->nlevels; ++m) p = child_begin(T, m, p);
    return p;
}

static void root_segment(const ora_tensor *T, int64_t *lo, int64_t *hi)
{
    const ora_level *l = &T->lvl[0];
    if (l->kind == ORA_COMPRESSED || l->kind == ORA_NONUNIQUE) { *lo = l->pos[0]; *hi = l->pos[1]; }
    else { *lo = 0; *hi = l->extent; }
}

/* Least position q in [lo, hi) whose coordinate is >= x; hi if none. */
static int64_t lower_bound(const int32_t *crd, int64_t lo, int64_t hi, int64_t x)
{
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if ((int64_t)crd[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

/* Position, inside the level-m segment [lo, hi) of T, of the first entry whose
 * coordinate is >= x (Dense: lo + x). */
static int64_t locate(const ora_tensor *T, int m, int64_t lo, int64_t hi, int64_t x)
{
    const ora_level *l = &T->lvl[m];
    if (l->kind != ORA_DENSE) return lower_bound(l->crd, lo, hi, x);   /* every sparse kind is sorted */
    (void)hi;
    return lo + x;
}

/* C_m(x | prefix) restricted to one operand: the number of its stored
 * non-zeros whose first m coordinates equal the prefix (that is the segment
 * [lo,hi) of level m) and whose level-m coordinate is < x  (Section 3.1 with
 * the cost of Section 4.2.2). */
static int64_t level_cost(const ora_tensor *T, int m, int64_t lo, int64_t hi, int64_t x)
{
    int64_t p = locate(T, m, lo, hi, x);
    return leaf_begin(T, m, p) - leaf_begin(T, m, lo);
}

int64_t ora_total_cost(const ora_tensor *ops, int k, int64_t tail_extent)
{
    int64_t w = tail_extent > 0 ? tail_extent : 1, q = 0;
    for (int t = 0; t < k; ++t) {
        int64_t lo, hi;
        root_segment(&ops[t], &lo, &hi);
        q += w * (leaf_begin(&ops[t], 0, hi) - leaf_begin(&ops[t], 0, lo));
    }
    return q;
}

/*
 * Algorithm 1, FindPartition(L, C, Q, N).
 *   ops[k]       coiterated operands, all with d levels over the same extents
 *   tail_extent  > 0: one more, dense, innermost loop of that extent below the
 *                d sparse levels, over which every operand is broadcast
 *                (SpMM's k loop); every stored non-zero then costs tail_extent
 *   Q            queried cost
 * Outputs: coord[d (+1 with a tail)], posn[k*d] (per operand t and level m, the
 * position of the first level-m entry that is not before the boundary),
 * *cost = C(x) = Q - final residual.
 */
int ora_find_partition(const ora_tensor *ops, int k, int d, int64_t tail_extent,
                       int64_t Q, int64_t *coord, int64_t *posn, int64_t *cost)
{
    if (k < 1 || k > ORA_MAXK || d < 1 || d > ORA_MAXL) return -1;
    int64_t w = tail_extent > 0 ? tail_extent : 1;
    int64_t lo[ORA_MAXK], hi[ORA_MAXK];
    int present[ORA_MAXK];
    int64_t R = Q;
    for (int t = 0; t < k; ++t) {
        if (ops[t].nlevels != d) return -1;
        root_segment(&ops[t], &lo[t], &hi[t]);
    }
    for (int m = 0; m < d; ++m) {
        int64_t N = ops[0].lvl[m].extent;
        /* HighestCoordinateLeqQuery: the largest x in [0, N] with C_m(x|.) <= R */
        int64_t low = 0, high = N;
        while (low < high) {
            int64_t x = low + (high - low + 1) / 2;
            int64_t c = 0;
            for (int t = 0; t < k; ++t) c += w * level_cost(&ops[t], m, lo[t], hi[t], x);
            if (c <= R) low = x; else high = x - 1;
        }
        int64_t xm = low, c = 0;
        for (int t = 0; t < k; ++t) c += w * level_cost(&ops[t], m, lo[t], hi[t], xm);
        R -= c;                                   /* residual inside the sub-space */
        coord[m] = xm;                            /* x <- x :: x_m                 */
        for (int t = 0; t < k; ++t) {
            const ora_tensor *T = &ops[t];
            int64_t p = locate(T, m, lo[t], hi[t], xm);
            posn[(size_t)t * d + m] = p;
            if (T->lvl[m].kind != ORA_DENSE)
                present[t] = (p < hi[t] && (int64_t)T->lvl[m].crd[p] == xm);
            else
                present[t] = (xm < N);
            if (m + 1 < d) {                      /* descend into x_m's children   */
                /* the positions that hold coordinate x_m: one, or (NONUNIQUE) all its repeats */
                int64_t p_end = present[t] ? p + 1 : p;
                if (T->lvl[m].kind == ORA_NONUNIQUE) p_end = lower_bound(T->lvl[m].crd, p, hi[t], xm + 1);
                lo[t] = child_begin(T, m, p);
                hi[t] = child_begin(T, m, p_end);
            }
        }
    }
    if (tail_extent > 0) {
        /* innermost dense loop: C_k(x | prefix) = x per operand storing prefix */
        int64_t np = 0;
        for (int t = 0; t < k; ++t) np += present[t];
        int64_t low = 0, high = tail_extent;
        while (low < high) {
            int64_t x = low + (high - low + 1) / 2;
            if (np * x <= R) low = x; else high = x - 1;
        }
        R -= np * low;
        coord[d] = low;
    }
    *cost = Q - R;
    return 0;
}

/* floor(p * total / P) without overflow. */
static int64_t equal_query(int64_t p, int64_t total, int64_t P)
{
    return (int64_t)(((__int128)p * (__int128)total) / (__int128)P);
}

/*
 * All P+1 boundaries of a P-way partition (Section 3.2: processor p searches
 * for p*Q/P and (p+1)*Q/P).  Boundary 0 is the origin and boundary P the end
 * of the iteration space by definition; interior boundaries come from
 * FindPartition, except that a query >= the total cost also yields the end.
 *   queries   NULL for equally spaced queries, else P+1 values (first and last
 *             are ignored)
 *   coord     [(P+1) * dc]  with dc = d + (tail_extent > 0)
 *   posn      [(P+1) * k * d]
 *   cost      [P+1]
 */
int ora_partition(const ora_tensor *ops, int k, int d, int64_t tail_extent, int64_t P,
                  const int64_t *queries, int64_t *coord, int64_t *posn, int64_t *cost)
{
    if (P < 1 || k < 1 || k > ORA_MAXK || d < 1 || d > ORA_MAXL) return -1;
    int dc = d + (tail_extent > 0 ? 1 : 0);
    int64_t total = ora_total_cost(ops, k, tail_extent);
    for (int64_t p = 0; p <= P; ++p) {
        int64_t *c = coord + (size_t)p * dc;
        int64_t *q = posn + (size_t)p * k * d;
        int64_t Q = queries ? queries[p] : equal_query(p, total, P);
        if (p == 0 || p == P || Q >= total) {
            int end = (p != 0);
            for (int m = 0; m < dc; ++m) c[m] = 0;
            if (end) c[0] = ops[0].lvl[0].extent;
            for (int t = 0; t < k; ++t) {
                int64_t lo, hi;
                root_segment(&ops[t], &lo, &hi);
                int64_t at = end ? hi : lo;
                for (int m = 0; m < d; ++m) {
                    q[(size_t)t * d + m] = at;
                    if (m + 1 < d) at = child_begin(&ops[t], m, at);
                }
            }
            cost[p] = end ? total : 0;
        } else {
            int rc = ora_find_partition(ops, k, d, tail_extent, Q, c, q, &cost[p]);
            if (rc) return rc;
        }
    }
    return 0;
}

/* ---- a row-aware cost function (variant) -------------------------------- */
/*
 * Section 4.2.2 counts stored non-zeros and remarks that this only approximates
 * the run time; a partition of 512 one-entry rows does more than one of a single
 * 512-entry row.  The variant below charges every level-0 position of an operand
 * (every row of a Dense level, every stored row of a Compressed one) `row_cost`
 * units on top of its stored non-zeros.  In the vocabulary of Section 3.1, for
 * two-level operands (i over j):
 *     C_i(x)     = sum_t [ non-zeros of t in rows before x  +  row_cost * (rows of t before x) ]
 *     C_j(x | i) = sum_{t storing row i} [ (x > 0 ? row_cost : 0)  +  entries of row i with column < x ]
 * Both are monotone, and C_j(N_j | i) = C_i(i + 1) - C_i(i): the pair is
 * hierarchically consistent, so Algorithm 1 applies unchanged.  The row's own
 * units sit in front of its first column: a boundary may fall at (i, 0).
 * FindPartition below is Algorithm 1 with these two functions, written out for
 * d = 2; outputs as ora_find_partition.
 */
static int64_t rows_before(const ora_tensor *T, int64_t lo, int64_t hi, int64_t x, int64_t *p_out)
{
    int64_t p = locate(T, 0, lo, hi, x);
    *p_out = p;
    return p - lo;
}

int64_t ora_total_cost_rowcost(const ora_tensor *ops, int k, int64_t row_cost)
{
    int64_t q = 0;
    for (int t = 0; t < k; ++t) {
        int64_t lo, hi;
        root_segment(&ops[t], &lo, &hi);
        q += leaf_begin(&ops[t], 0, hi) - leaf_begin(&ops[t], 0, lo) + row_cost * (hi - lo);
    }
    return q;
}

int ora_find_partition_rowcost(const ora_tensor *ops, int k, int64_t row_cost, int64_t Q,
                               int64_t *coord, int64_t *posn, int64_t *cost)
{
    if (k < 1 || k > ORA_MAXK || row_cost < 0) return -1;
    int64_t lo[ORA_MAXK], hi[ORA_MAXK];
    int present[ORA_MAXK];
    int64_t R = Q;
    for (int t = 0; t < k; ++t) {
        if (ops[t].nlevels != 2) return -1;
        root_segment(&ops[t], &lo[t], &hi[t]);
    }
    /* level 0: the highest row x with C_i(x) <= R */
    {
        int64_t N = ops[0].lvl[0].extent, low = 0, high = N;
        while (low < high) {
            int64_t x = low + (high - low + 1) / 2, c = 0, p;
            for (int t = 0; t < k; ++t)
                c += level_cost(&ops[t], 0, lo[t], hi[t], x) + row_cost * rows_before(&ops[t], lo[t], hi[t], x, &p);
            if (c <= R) low = x; else high = x - 1;
        }
        int64_t x0 = low, c = 0, p;
        for (int t = 0; t < k; ++t)
            c += level_cost(&ops[t], 0, lo[t], hi[t], x0) + row_cost * rows_before(&ops[t], lo[t], hi[t], x0, &p);
        R -= c;
        coord[0] = x0;
        for (int t = 0; t < k; ++t) {
            const ora_tensor *T = &ops[t];
            rows_before(T, lo[t], hi[t], x0, &p);
            posn[(size_t)t * 2 + 0] = p;
            if (T->lvl[0].kind != ORA_DENSE) present[t] = (p < hi[t] && (int64_t)T->lvl[0].crd[p] == x0);
            else present[t] = (x0 < N);
            lo[t] = child_begin(T, 0, p);
            hi[t] = child_begin(T, 0, present[t] ? p + 1 : p);
        }
    }
    /* level 1: the highest column x with C_j(x | row) <= R */
    {
        int64_t N = ops[0].lvl[1].extent, low = 0, high = N;
        while (low < high) {
            int64_t x = low + (high - low + 1) / 2, c = 0;
            for (int t = 0; t < k; ++t)
                if (present[t]) c += (x > 0 ? row_cost : 0) + level_cost(&ops[t], 1, lo[t], hi[t], x);
            if (c <= R) low = x; else high = x - 1;
        }
        int64_t x1 = low, c = 0;
        for (int t = 0; t < k; ++t)
            if (present[t]) c += (x1 > 0 ? row_cost : 0) + level_cost(&ops[t], 1, lo[t], hi[t], x1);
        R -= c;
        coord[1] = x1;
        for (int t = 0; t < k; ++t) posn[(size_t)t * 2 + 1] = locate(&ops[t], 1, lo[t], hi[t], x1);
    }
    *cost = Q - R;
    return 0;
}

/* All P+1 boundaries with the row-aware cost; conventions of ora_partition. */
int ora_partition_rowcost(const ora_tensor *ops, int k, int64_t row_cost, int64_t P, const int64_t *queries,
                          int64_t *coord, int64_t *posn, int64_t *cost)
{
    if (P < 1 || k < 1 || k > ORA_MAXK) return -1;
    int64_t total = ora_total_cost_rowcost(ops, k, row_cost);
    for (int64_t p = 0; p <= P; ++p) {
        int64_t *c = coord + (size_t)p * 2;
        int64_t *q = posn + (size_t)p * k * 2;
        int64_t Q = queries ? queries[p] : equal_query(p, total, P);
        if (p == 0 || p == P || Q >= total) {
            int end = (p != 0);
            c[0] = end ? ops[0].lvl[0].extent : 0;
            c[1] = 0;
            for (int t = 0; t < k; ++t) {
                int64_t lo, hi;
                root_segment(&ops[t], &lo, &hi);
                int64_t at = end ? hi : lo;
                q[(size_t)t * 2 + 0] = at;
                q[(size_t)t * 2 + 1] = child_begin(&ops[t], 0, at);
            }
            cost[p] = end ? total : 0;
        } else {
            int rc = ora_find_partition_rowcost(ops, k, row_cost, Q, c, q, &cost[p]);
            if (rc) return rc;
        }
    }
    return 0;
}

/* ---- plain definitions of the balanced kernels -------------------------- */

/* y_i = sum_j A_ij x_j, CSR, fp64 inputs, long double accumulation.
 * s_i = sum_j |A_ij x_j| (for the tolerance rule). */
void ora_spmv_f64(int64_t n_rows, const int32_t *pos, const int32_t *crd, const double *val,
                  const double *x, double *y, double *s)
{
    for (int64_t i = 0; i < n_rows; ++i) {
        long double acc = 0.0L, sabs = 0.0L;
        for (int64_t q = pos[i]; q < pos[i + 1]; ++q) {
            long double term = (long double)val[q] * (long double)x[crd[q]];
            acc += term;
            sabs += fabsl(term);
        }
        y[i] = (double)acc;
        if (s) s[i] = (double)sabs;
    }
}

/* Same for fp32 inputs, double accumulation, double outputs. */
void ora_spmv_f32(int64_t n_rows, const int32_t *pos, const int32_t *crd, const float *val,
                  const float *x, double *y, double *s)
{
    for (int64_t i = 0; i < n_rows; ++i) {
        double acc = 0.0, sabs = 0.0;
        for (int64_t q = pos[i]; q < pos[i + 1]; ++q) {
            double term = (double)val[q] * (double)x[crd[q]];
            acc += term;
            sabs += fabs(term);
        }
        y[i] = acc;
        if (s) s[i] = sabs;
    }
}

/* C_ik = sum_j A_ij B_jk; A CSR fp32, B dense row-major [*, n] with leading
 * dimension ldb, C and S (sum of |terms|) dense double [n_rows, n]. */
void ora_spmm_f32(int64_t n_rows, const int32_t *pos, const int32_t *crd, const float *val,
                  const float *B, int64_t n, int64_t ldb, double *C, double *S)
{
    for (int64_t i = 0; i < n_rows; ++i) {
        double *c = C + (size_t)i * n;
        double *s = S ? S + (size_t)i * n : NULL;
        for (int64_t kk = 0; kk < n; ++kk) { c[kk] = 0.0; if (s) s[kk] = 0.0; }
        for (int64_t q = pos[i]; q < pos[i + 1]; ++q) {
            const float *b = B + (size_t)crd[q] * ldb;
            double a = (double)val[q];
            for (int64_t kk = 0; kk < n; ++kk) {
                double term = a * (double)b[kk];
                c[kk] += term;
                if (s) s[kk] += fabs(term);
            }
        }
    }
}

void ora_spmm_f64(int64_t n_rows, const int32_t *pos, const int32_t *crd, const double *val,
                  const double *B, int64_t n, int64_t ldb, double *C, double *S)
{
    for (int64_t i = 0; i < n_rows; ++i) {
        for (int64_t kk = 0; kk < n; ++kk) {
            long double acc = 0.0L, sabs = 0.0L;
            for (int64_t q = pos[i]; q < pos[i + 1]; ++q) {
                long double term = (long double)val[q] * (long double)B[(size_t)crd[q] * ldb + kk];
                acc += term;
                sabs += fabsl(term);
            }
            C[(size_t)i * n + kk] = (double)acc;
            if (S) S[(size_t)i * n + kk] = (double)sabs;
        }
    }
}

static double load_value(const void *val, int is_f64, int64_t q)
{
    return is_f64 ? ((const double *)val)[q] : (double)((const float *)val)[q];
}

/*
 * k-finger union merge of the segments [p[t], e[t]) of k sorted coordinate
 * lists (the coiteration loop of Section 2.1 with "any" for "all").  Appends to
 * out_crd/out_val/out_abs at *n_out.  Values are added in operand order.
 */
static void union_merge(int k, const int32_t *const *crd, const void *const *val, int is_f64,
                        int64_t *p, const int64_t *e,
                        int32_t *out_crd, double *out_val, double *out_abs, int64_t *n_out)
{
    for (;;) {
        int any = 0;
        int64_t i = 0;
        for (int t = 0; t < k; ++t)
            if (p[t] < e[t]) {
                int64_t it = crd[t][p[t]];
                if (!any || it < i) i = it;
                any = 1;
            }
        if (!any) break;
        double sum = 0.0, sabs = 0.0;
        for (int t = 0; t < k; ++t)
            if (p[t] < e[t] && (int64_t)crd[t][p[t]] == i) {
                double v = load_value(val[t], is_f64, p[t]);
                sum += v;
                sabs += fabs(v);
                ++p[t];
            }
        out_crd[*n_out] = (int32_t)i;
        out_val[*n_out] = sum;
        if (out_abs) out_abs[*n_out] = sabs;
        ++*n_out;
    }
}

/* z = sum_t v_t for k sparse vectors (sorted unique indices).  Outputs must
 * hold sum_t nnz_t entries; returns the number written. */
int64_t ora_spadd_vec(int k, const int32_t *const *idx, const void *const *val, const int64_t *nnz,
                      int is_f64, int32_t *out_idx, double *out_val, double *out_abs)
{
    int64_t p[ORA_MAXK], n_out = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    for (int t = 0; t < k; ++t) p[t] = 0;
    union_merge(k, idx, val, is_f64, p, nnz, out_idx, out_val, out_abs, &n_out);
    return n_out;
}

/*
 * Z = sum_t A_t for k DCSR matrices (Section 2.2: rows coiterated as a union,
 * then the columns of the operands that store the row).  out_crd0/out_pos1 must
 * hold sum_t rows_t (+1) entries, out_crd1/out_val sum_t nnz_t.  counts[0] =
 * stored rows, counts[1] = nnz of Z.  out_pos0 = {0, rows}.
 */
int ora_spadd_dcsr(int k, const int32_t *const *pos0, const int32_t *const *crd0,
                   const int32_t *const *pos1, const int32_t *const *crd1,
                   const void *const *val, int is_f64,
                   int32_t *out_pos0, int32_t *out_crd0, int32_t *out_pos1, int32_t *out_crd1,
                   double *out_val, double *out_abs, int64_t *counts)
{
    int64_t r[ORA_MAXK], re[ORA_MAXK], p[ORA_MAXK], e[ORA_MAXK];
    int64_t nr = 0, nz = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    for (int t = 0; t < k; ++t) { r[t] = pos0[t][0]; re[t] = pos0[t][1]; }
    out_pos1[0] = 0;
    for (;;) {
        int any = 0;
        int64_t i = 0;
        for (int t = 0; t < k; ++t)
            if (r[t] < re[t]) {
                int64_t it = crd0[t][r[t]];
                if (!any || it < i) i = it;
                any = 1;
            }
        if (!any) break;
        for (int t = 0; t < k; ++t) {
            if (r[t] < re[t] && (int64_t)crd0[t][r[t]] == i) {
                p[t] = pos1[t][r[t]];
                e[t] = pos1[t][r[t] + 1];
                ++r[t];
            } else {
                p[t] = e[t] = 0;
            }
        }
        int64_t before = nz;
        union_merge(k, crd1, val, is_f64, p, e, out_crd1, out_val, out_abs, &nz);
        if (nz > before) {                 /* a stored row holds at least one entry */
            out_crd0[nr] = (int32_t)i;
            out_pos1[nr + 1] = (int32_t)nz;
            ++nr;
        }
    }
    out_pos0[0] = 0;
    out_pos0[1] = (int32_t)nr;
    counts[0] = nr;
    counts[1] = nz;
    return 0;
}

/*
 * Z = sum_t A_t for k CSR matrices with the same shape (dense rows, union of
 * the columns per row).  out_pos has n_rows+1 entries.  Returns nnz of Z.
 */
int64_t ora_spadd_csr(int k, int64_t n_rows, const int32_t *const *pos, const int32_t *const *crd,
                      const void *const *val, int is_f64,
                      int32_t *out_pos, int32_t *out_crd, double *out_val, double *out_abs)
{
    int64_t p[ORA_MAXK], e[ORA_MAXK], nz = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    out_pos[0] = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        for (int t = 0; t < k; ++t) { p[t] = pos[t][i]; e[t] = pos[t][i + 1]; }
        union_merge(k, crd, val, is_f64, p, e, out_crd, out_val, out_abs, &nz);
        out_pos[i + 1] = (int32_t)nz;
    }
    return nz;
}

/*
 * k-finger intersection of the segments [p[t], e[t]) of k sorted coordinate
 * lists: the sequential loop of Section 2.1 (z_i = a_i b_i c_i): while every
 * finger is inside its segment, take the smallest coordinate under the
 * fingers; if all fingers show it, emit the product; advance every finger that
 * shows it.  Appends to out_crd/out_val/out_abs at *n_out.
 */
static void intersect_merge(int k, const int32_t *const *crd, const void *const *val, int is_f64,
                            int64_t *p, const int64_t *e,
                            int32_t *out_crd, double *out_val, double *out_abs, int64_t *n_out)
{
    for (;;) {
        int inside = 1;
        for (int t = 0; t < k; ++t)
            if (p[t] >= e[t]) inside = 0;
        if (!inside) break;
        int64_t i = crd[0][p[0]];
        for (int t = 1; t < k; ++t)
            if ((int64_t)crd[t][p[t]] < i) i = crd[t][p[t]];
        int all = 1;
        for (int t = 0; t < k; ++t)
            if ((int64_t)crd[t][p[t]] != i) all = 0;
        if (all) {
            double prod = 1.0;
            for (int t = 0; t < k; ++t) prod *= load_value(val[t], is_f64, p[t]);
            out_crd[*n_out] = (int32_t)i;
            out_val[*n_out] = prod;
            if (out_abs) out_abs[*n_out] = fabs(prod);
            ++*n_out;
        }
        for (int t = 0; t < k; ++t)
            if ((int64_t)crd[t][p[t]] == i) ++p[t];
    }
}

/* z_i = prod_t v_t,i over the coordinates all k sparse vectors store.  Outputs
 * must hold min_t nnz_t entries; returns the number written. */
int64_t ora_spmul_vec(int k, const int32_t *const *idx, const void *const *val, const int64_t *nnz,
                      int is_f64, int32_t *out_idx, double *out_val, double *out_abs)
{
    int64_t p[ORA_MAXK], n_out = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    for (int t = 0; t < k; ++t) p[t] = 0;
    intersect_merge(k, idx, val, is_f64, p, nnz, out_idx, out_val, out_abs, &n_out);
    return n_out;
}

/* Z_ij = prod_t A_t,ij (Hadamard product) of k CSR matrices of one shape: dense
 * rows, intersection of the columns per row.  Returns nnz of Z. */
int64_t ora_spmul_csr(int k, int64_t n_rows, const int32_t *const *pos, const int32_t *const *crd,
                      const void *const *val, int is_f64,
                      int32_t *out_pos, int32_t *out_crd, double *out_val, double *out_abs)
{
    int64_t p[ORA_MAXK], e[ORA_MAXK], nz = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    out_pos[0] = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        for (int t = 0; t < k; ++t) { p[t] = pos[t][i]; e[t] = pos[t][i + 1]; }
        intersect_merge(k, crd, val, is_f64, p, e, out_crd, out_val, out_abs, &nz);
        out_pos[i + 1] = (int32_t)nz;
    }
    return nz;
}

/* ---- nested intersections: Section 3.3 ---------------------------------- */

/*
 * Z_ij = prod_t A_t,ij for k DCSR matrices: the loop nest of Section 3.3
 * (rows coiterated as an INTERSECTION, then the columns of the row as an
 * intersection), serially.  As in the union, a row is stored only when it
 * holds at least one entry.  out_crd0/out_pos1 must hold min_t rows_t (+1)
 * entries, out_crd1/out_val min_t nnz_t.  counts = {stored rows, nnz}.
 */
int ora_spmul_dcsr(int k, const int32_t *const *pos0, const int32_t *const *crd0,
                   const int32_t *const *pos1, const int32_t *const *crd1,
                   const void *const *val, int is_f64,
                   int32_t *out_pos0, int32_t *out_crd0, int32_t *out_pos1, int32_t *out_crd1,
                   double *out_val, double *out_abs, int64_t *counts)
{
    int64_t r[ORA_MAXK], re[ORA_MAXK], p[ORA_MAXK], e[ORA_MAXK];
    int64_t nr = 0, nz = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    for (int t = 0; t < k; ++t) { r[t] = pos0[t][0]; re[t] = pos0[t][1]; }
    out_pos1[0] = 0;
    for (;;) {
        int inside = 1;
        for (int t = 0; t < k; ++t)
            if (r[t] >= re[t]) inside = 0;
        if (!inside) break;
        int64_t i = crd0[0][r[0]];
        for (int t = 1; t < k; ++t)
            if ((int64_t)crd0[t][r[t]] < i) i = crd0[t][r[t]];
        int all = 1;
        for (int t = 0; t < k; ++t)
            if ((int64_t)crd0[t][r[t]] != i) all = 0;
        if (all) {
            for (int t = 0; t < k; ++t) { p[t] = pos1[t][r[t]]; e[t] = pos1[t][r[t] + 1]; }
            int64_t before = nz;
            intersect_merge(k, crd1, val, is_f64, p, e, out_crd1, out_val, out_abs, &nz);
            if (nz > before) {
                out_crd0[nr] = (int32_t)i;
                out_pos1[nr + 1] = (int32_t)nz;
                ++nr;
            }
        }
        for (int t = 0; t < k; ++t)
            if ((int64_t)crd0[t][r[t]] == i) ++r[t];
    }
    out_pos0[0] = 0;
    out_pos0[1] = (int32_t)nr;
    counts[0] = nr;
    counts[1] = nz;
    return 0;
}

/*
 * First loop of the rewritten nest of Section 3.3 ("Efficiently computing
 * remapped cost functions"): coiterate the rows all k operands store and, for
 * every such row i (the i'-th one), memoise
 *     T[i'] = C_j(N_j | i) = sum_t (number of entries operand t stores in row i).
 * Also returns the row coordinate rows[i'] and, per operand, the position
 * rpos[t * cap + i'] of the row in the operand's level 0.  Arrays hold cap >=
 * min_t rows_t entries.  Returns the number M of intersected rows.
 */
int64_t ora_remap_rows(int k, const int32_t *const *pos0, const int32_t *const *crd0,
                       const int32_t *const *pos1, int64_t cap,
                       int64_t *rows, int64_t *rpos, int64_t *T)
{
    int64_t r[ORA_MAXK], re[ORA_MAXK], M = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    for (int t = 0; t < k; ++t) { r[t] = pos0[t][0]; re[t] = pos0[t][1]; }
    for (;;) {
        int inside = 1;
        for (int t = 0; t < k; ++t)
            if (r[t] >= re[t]) inside = 0;
        if (!inside) break;
        int64_t i = crd0[0][r[0]];
        for (int t = 1; t < k; ++t)
            if ((int64_t)crd0[t][r[t]] < i) i = crd0[t][r[t]];
        int all = 1;
        for (int t = 0; t < k; ++t)
            if ((int64_t)crd0[t][r[t]] != i) all = 0;
        if (all) {
            if (M >= cap) return -1;
            int64_t c = 0;
            for (int t = 0; t < k; ++t) {
                c += pos1[t][r[t] + 1] - pos1[t][r[t]];
                rpos[(size_t)t * cap + M] = r[t];
            }
            rows[M] = i;
            T[M] = c;
            ++M;
        }
        for (int t = 0; t < k; ++t)
            if ((int64_t)crd0[t][r[t]] == i) ++r[t];
    }
    return M;
}

/*
 * FindRecursivePartition (Algorithm 2) for the Hadamard product of k DCSR
 * matrices.  The outermost sparse intersection (the row loop) is not the
 * innermost loop, so its cost function is remapped: the row loop becomes a
 * loop over i' in [0, M), the intersected rows, with
 *     C'_i(x) = T'[x],   T' = exclusive prefix sum of T          (Section 3.3)
 * and the remapped nest (i' dense, then the column intersection, which is
 * innermost and needs no remapping) is handed to FindPartition (Algorithm 1)
 * with the cost of Section 4.2.2.
 *
 * Inputs: the operands, M, rpos and T from ora_remap_rows (cap = stride of
 * rpos), n_cols, P, optional queries (P + 1, as in ora_partition).
 * Outputs per boundary b (boundary 0 = origin, boundary P = end of the
 * remapped space, by the same definition as ora_partition):
 *   coord[b*2 + {0,1}]            (i', j)
 *   lpos[(b*k + t)]               position in operand t's crd1/val of its first
 *                                 entry of row i' that is not before j
 *                                 (for i' == M: one past its last entry of row M-1,
 *                                 or its pos1[0] when M == 0)
 *   before[(b*k + t)]             number of entries operand t stores in the
 *                                 intersected rows before the boundary
 *   cost[b]                       C(boundary) = sum_t before
 * Tprime must hold M + 1 entries and returns T'.
 */
int ora_recursive_partition_dcsr(int k, const int32_t *const *pos1, const int32_t *const *crd1,
                                 int64_t n_cols, int64_t M, int64_t cap, const int64_t *rpos,
                                 const int64_t *T, int64_t P, const int64_t *queries,
                                 int64_t *Tprime, int64_t *coord, int64_t *lpos, int64_t *before,
                                 int64_t *cost)
{
    if (k < 1 || k > ORA_MAXK || P < 1 || M < 0) return -1;
    Tprime[0] = 0;
    for (int64_t x = 0; x < M; ++x) Tprime[x + 1] = Tprime[x] + T[x];
    const int64_t total = Tprime[M];
    /* per operand: entries stored in the intersected rows before row y (for `before`) */
    int64_t *rows_before = (int64_t *)malloc(sizeof(int64_t) * (size_t)k * (size_t)(M + 1));
    if (!rows_before) return -1;
    for (int t = 0; t < k; ++t) {
        int64_t *s = rows_before + (size_t)t * (M + 1);
        s[0] = 0;
        for (int64_t y = 0; y < M; ++y) {
            int64_t q = rpos[(size_t)t * cap + y];
            s[y + 1] = s[y] + (pos1[t][q + 1] - pos1[t][q]);
        }
    }
    for (int64_t b = 0; b <= P; ++b) {
        int64_t Q = queries ? queries[b] : equal_query(b, total, P);
        int64_t x, j = 0, R;
        if (b == 0) { x = 0; R = 0; Q = 0; }
        else if (b == P || Q >= total) { x = M; R = 0; Q = total; }
        else {
            /* level i': highest x in [0, M] with C'_i(x) = T'[x] <= Q */
            int64_t low = 0, high = M;
            while (low < high) {
                int64_t mid = low + (high - low + 1) / 2;
                if (Tprime[mid] <= Q) low = mid; else high = mid - 1;
            }
            x = low;
            R = Q - Tprime[x];
            /* level j inside row x: highest j in [0, N_j] with C_j(j | x) <= R */
            int64_t lowj = 0, highj = n_cols;
            while (lowj < highj) {
                int64_t mid = lowj + (highj - lowj + 1) / 2;
                int64_t c = 0;
                for (int t = 0; t < k; ++t) {
                    int64_t q = rpos[(size_t)t * cap + x];
                    c += lower_bound(crd1[t], pos1[t][q], pos1[t][q + 1], mid) - pos1[t][q];
                }
                if (c <= R) lowj = mid; else highj = mid - 1;
            }
            j = lowj;
        }
        coord[b * 2 + 0] = x;
        coord[b * 2 + 1] = j;
        int64_t csum = 0;
        for (int t = 0; t < k; ++t) {
            int64_t at, bef = rows_before[(size_t)t * (M + 1) + x];
            if (x < M) {
                int64_t q = rpos[(size_t)t * cap + x];
                at = lower_bound(crd1[t], pos1[t][q], pos1[t][q + 1], j);
                bef += at - pos1[t][q];
            } else if (M > 0) {
                at = pos1[t][rpos[(size_t)t * cap + M - 1] + 1];
            } else {
                at = pos1[t][0];
            }
            lpos[b * k + t] = at;
            before[b * k + t] = bef;
            csum += bef;
        }
        cost[b] = csum;
        (void)R;
    }
    free(rows_before);
    return 0;
}


/* ---- coordinate-list (COO) matrices ---------------------------------------- */

/* Union add / intersection multiply of k COO matrices (rows[t], cols[t] sorted by (row, col),
 * no repeated pair): the k-finger coiteration of Section 2.1 over coordinate PAIRS, "any" for the
 * sum and "all" for the product, values combined in operand order.  Outputs hold sum_t nnz_t
 * (add) or min_t nnz_t (multiply) entries; returns the number written. */
static int64_t coo_merge(int multiply, int k, const int32_t *const *rows, const int32_t *const *cols,
                         const void *const *val, const int64_t *nnz, int is_f64,
                         int32_t *out_row, int32_t *out_col, double *out_val, double *out_abs)
{
    int64_t p[ORA_MAXK], n_out = 0;
    if (k < 1 || k > ORA_MAXK) return -1;
    for (int t = 0; t < k; ++t) p[t] = 0;
    for (;;) {
        int any = 0, all = 1;
        int64_t bi = 0, bj = 0;
        for (int t = 0; t < k; ++t) {
            if (p[t] >= nnz[t]) { all = 0; continue; }
            int64_t i = rows[t][p[t]], j = cols[t][p[t]];
            if (!any || i < bi || (i == bi && j < bj)) { bi = i; bj = j; }
            any = 1;
        }
        if (!any || (multiply && !all)) break;      /* a product ends with its first exhausted operand */
        double acc = multiply ? 1.0 : 0.0, sabs = 0.0;
        int holders = 0;
        for (int t = 0; t < k; ++t)
            if (p[t] < nnz[t] && rows[t][p[t]] == bi && cols[t][p[t]] == bj) {
                double v = load_value(val[t], is_f64, p[t]);
                if (multiply) acc *= v; else { acc += v; sabs += fabs(v); }
                ++holders;
            }
        if (!multiply || holders == k) {
            out_row[n_out] = (int32_t)bi;
            out_col[n_out] = (int32_t)bj;
            out_val[n_out] = acc;
            if (out_abs) out_abs[n_out] = multiply ? fabs(acc) : sabs;
            ++n_out;
        }
        for (int t = 0; t < k; ++t)
            if (p[t] < nnz[t] && rows[t][p[t]] == bi && cols[t][p[t]] == bj) ++p[t];
    }
    return n_out;
}

int64_t ora_spadd_coo(int k, const int32_t *const *rows, const int32_t *const *cols,
                      const void *const *val, const int64_t *nnz, int is_f64,
                      int32_t *out_row, int32_t *out_col, double *out_val, double *out_abs)
{
    return coo_merge(0, k, rows, cols, val, nnz, is_f64, out_row, out_col, out_val, out_abs);
}

int64_t ora_spmul_coo(int k, const int32_t *const *rows, const int32_t *const *cols,
                      const void *const *val, const int64_t *nnz, int is_f64,
                      int32_t *out_row, int32_t *out_col, double *out_val, double *out_abs)
{
    return coo_merge(1, k, rows, cols, val, nnz, is_f64, out_row, out_col, out_val, out_abs);
}

/* ---- union addition of third-order tensors (three compressed levels, CSF) ---- */
/*
 * Z_ijk = sum_t T^t_ijk over the union of the operands' stored coordinates: the
 * coiteration nest of Section 2.2 one level deeper.  At every level the fingers of
 * the operands that store the prefix walk their segments; the smallest coordinate
 * under a finger is emitted ("any operand matches"), and the operands that hold it
 * descend into their child segments.  Values of coinciding entries are added in
 * operand order.  The result is CSF as well: crd0 / pos1 / crd1 / pos2 / crd2 / val.
 */
typedef struct {
    int k, is_f64;
    const int32_t *const *pos[3];
    const int32_t *const *crd[3];
    const void *const *val;
    int32_t *ocrd[3];
    int32_t *opos[3];        /* opos[m][c] = first child (level m) of output entry c of level m - 1 */
    double *oval, *oabs;
    int64_t n[3];
} csf3_ctx;

static void csf3_coiterate(csf3_ctx *c, int m, const int64_t *lo, const int64_t *hi)
{
    int64_t f[ORA_MAXK], clo[ORA_MAXK], chi[ORA_MAXK];
    for (int t = 0; t < c->k; ++t) f[t] = lo[t];
    for (;;) {
        int64_t x = INT64_MAX;
        for (int t = 0; t < c->k; ++t)
            if (f[t] < hi[t] && (int64_t)c->crd[m][t][f[t]] < x) x = c->crd[m][t][f[t]];
        if (x == INT64_MAX) break;
        c->ocrd[m][c->n[m]] = (int32_t)x;
        if (m < 2) {
            c->opos[m + 1][c->n[m]] = (int32_t)c->n[m + 1];
            for (int t = 0; t < c->k; ++t) {
                if (f[t] < hi[t] && (int64_t)c->crd[m][t][f[t]] == x) {
                    clo[t] = c->pos[m + 1][t][f[t]];
                    chi[t] = c->pos[m + 1][t][f[t] + 1];
                    ++f[t];
                } else {
                    clo[t] = chi[t] = 0;
                }
            }
            ++c->n[m];
            csf3_coiterate(c, m + 1, clo, chi);
        } else {
            double sum = 0.0, sabs = 0.0;
            for (int t = 0; t < c->k; ++t)
                if (f[t] < hi[t] && (int64_t)c->crd[m][t][f[t]] == x) {
                    double v = load_value(c->val[t], c->is_f64, f[t]);
                    sum += v;
                    sabs += fabs(v);
                    ++f[t];
                }
            c->oval[c->n[2]] = sum;
            c->oabs[c->n[2]] = sabs;
            ++c->n[2];
        }
    }
}

/* counts[3] = stored coordinates of the result at levels 0, 1, 2 */
int ora_spadd_csf3(int k, const int32_t *const *pos0, const int32_t *const *crd0, const int32_t *const *pos1,
                   const int32_t *const *crd1, const int32_t *const *pos2, const int32_t *const *crd2,
                   const void *const *val, int is_f64, int32_t *opos0, int32_t *ocrd0, int32_t *opos1,
                   int32_t *ocrd1, int32_t *opos2, int32_t *ocrd2, double *oval, double *oabs, int64_t *counts)
{
    if (k < 1 || k > ORA_MAXK) return -1;
    csf3_ctx c;
    c.k = k; c.is_f64 = is_f64;
    c.pos[0] = pos0; c.pos[1] = pos1; c.pos[2] = pos2;
    c.crd[0] = crd0; c.crd[1] = crd1; c.crd[2] = crd2;
    c.val = val;
    c.ocrd[0] = ocrd0; c.ocrd[1] = ocrd1; c.ocrd[2] = ocrd2;
    c.opos[0] = opos0; c.opos[1] = opos1; c.opos[2] = opos2;
    c.oval = oval; c.oabs = oabs;
    c.n[0] = c.n[1] = c.n[2] = 0;
    int64_t lo[ORA_MAXK], hi[ORA_MAXK];
    for (int t = 0; t < k; ++t) { lo[t] = pos0[t][0]; hi[t] = pos0[t][1]; }
    csf3_coiterate(&c, 0, lo, hi);
    opos0[0] = 0;
    opos0[1] = (int32_t)c.n[0];
    opos1[c.n[0]] = (int32_t)c.n[1];
    opos2[c.n[1]] = (int32_t)c.n[2];
    counts[0] = c.n[0]; counts[1] = c.n[1]; counts[2] = c.n[2];
    return 0;
}

/* Timing aid for benchmarks (no arithmetic of its own): runs ora_spmv_f64 `reps`
 * times and returns the shortest duration in seconds, measured with the
 * monotonic clock around the call. */
#include <time.h>
double ora_time_spmv_f64(int64_t n_rows, const int32_t *pos, const int32_t *crd, const double *val,
                         const double *x, double *y, double *s, int32_t reps)
{
    double best = -1.0;
    for (int32_t r = 0; r < reps; ++r) {
        struct timespec a, b;
        clock_gettime(CLOCK_MONOTONIC, &a);
        ora_spmv_f64(n_rows, pos, crd, val, x, y, s);
        clock_gettime(CLOCK_MONOTONIC, &b);
        double t = (double)(b.tv_sec - a.tv_sec) + 1e-9 * (double)(b.tv_nsec - a.tv_nsec);
        if (best < 0.0 || t < best) best = t;
    }
    return best;
}
