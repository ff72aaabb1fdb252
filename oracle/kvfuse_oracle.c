/*
 * kvfuse_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, single-threaded CPU statement of Fast Fusion (the paper's
 * Algorithm 1 and the method section around it) for ONE group of KV blocks,
 * i.e. one (layer, KV head).  Every floating-point step is done in fp64 with
 * one accumulator and left-to-right order; nothing is blocked, fused or
 * vectorised by hand.  It shares no code, header, table or constant with the
 * HIP library; only tests, the smoke check and the CPU-baseline leg of the
 * benchmark may call it.
 *
 * Readings of the paper taken here (all listed again in the design notes):
 *   - A "block vector" is the r = t*d values of one block of one KV head
 *     (method section: the cache is unfolded to one r-vector per block).
 *   - Leaf step of Algorithm 1 ("normalize"): the norm of every block is
 *     stored; the raw block stays in the pool and its unit direction is
 *     x / ||x|| whenever Algorithm 1 needs it.  A block of norm 0 has the
 *     zero vector as direction and similarity 0 with everything.
 *   - Similarity line of Algorithm 1: sim = k_l k_r^T on unit vectors, keys
 *     only, computed once per tree node before any row of k_l is changed.
 *   - Threshold line: strict '>'.  A right block that clears the threshold
 *     for several left rows goes to the row with the largest similarity, the
 *     lowest row index winning exact ties (a block-table entry can point at
 *     one physical block only).
 *   - Fusion lines: k_l(row) <- normalize(k_l(row) + sum of fused k_r rows),
 *     operands being the CURRENT unit representatives; v follows with the
 *     same index set.  The result is rounded to the pool's storage type when
 *     it is written back and its norm is recomputed from the rounded values.
 *   - "evict", "update block-table": every logical block that pointed at an
 *     evicted right block now points at the left row's physical block; the
 *     evicted id goes to the free list; reference counts add up.
 *   - Return line: survivors are k_l followed by the non-fused rows of k_r in
 *     their original order.
 *   - Method section, "norm of each r is stored to allow a proper rescaling":
 *     logical block x is represented as scale[x] * stored(bt[x]) with
 *     scale[x] = ||original x|| / ||stored(bt[x])||.
 *
 * Storage types: elem_bytes == 4 -> IEEE binary32, elem_bytes == 2 ->
 * bfloat16 (upper 16 bits of a binary32), both little endian.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* storage type helpers                                                */
/* ------------------------------------------------------------------ */

static double ora_load(const void *base, int elem_bytes, size_t idx)
{
    if (elem_bytes == 4) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
}

/* Round a finite double to the nearest bfloat16 (ties to even) without going
 * through binary32 first, so there is no double rounding: scale so that one
 * unit in the last place of the target is 1.0, round to the nearest integer
 * with rint() (default rounding mode = ties to even), scale back. */
static double ora_round_to_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x))
        return x;
    int e;
    (void)frexp(fabs(x), &e); /* |x| = m * 2^e, 0.5 <= m < 1 */
    int q = e - 8;            /* 8 significant bits: ulp = 2^(e-8) */
    if (q < -133)
        q = -133;             /* subnormal range: fixed ulp 2^-133 */
    double y = ldexp(rint(ldexp(x, -q)), q);
    if (fabs(y) > 3.3895313892515355e38) /* largest finite bfloat16 */
        y = (x > 0) ? INFINITY : -INFINITY;
    return y;
}

static void ora_store(void *base, int elem_bytes, size_t idx, double x)
{
    if (elem_bytes == 4) {
        ((float *)base)[idx] = (float)x; /* C conversion: round to nearest even */
    } else {
        float f = (float)ora_round_to_bf16(x); /* exact: value is a bfloat16 */
        uint32_t bits;
        memcpy(&bits, &f, 4);
        ((uint16_t *)base)[idx] = (uint16_t)(bits >> 16);
    }
}

/* exported so that tests can pin the rounding rule on its own */
double ora_test_round_bf16(double x) { return ora_round_to_bf16(x); }

/* n doubles -> n values of the pool's storage type (float, or bfloat16 bit patterns), one rounding each */
void ora_store_array(void *dst, int elem_bytes, const double *x, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        ora_store(dst, elem_bytes, i, x[i]);
}

/* ------------------------------------------------------------------ */
/* the steps of one tree node                                          */
/* ------------------------------------------------------------------ */

/* Method section: every block vector keeps its norm.  norm[b] = ||block b||_2 of
 * the values as stored, for blocks 0..P-1 of one pool tensor [P][r]. */
void ora_block_norms(const void *pool, int elem_bytes, int r, int P, double *norm)
{
    for (int b = 0; b < P; ++b) {
        double ss = 0.0;
        for (int e = 0; e < r; ++e) {
            double x = ora_load(pool, elem_bytes, (size_t)b * r + e);
            ss += x * x;
        }
        norm[b] = sqrt(ss);
    }
}

/* One entry of sim = k_l k_r^T (Algorithm 1, similarity line) for physical
 * blocks a and b: cosine of the stored vectors. */
static double ora_cosine(const void *pool, int elem_bytes, int r, const double *norm, int a, int b)
{
    if (norm[a] == 0.0 || norm[b] == 0.0)
        return 0.0;
    double dot = 0.0;
    for (int e = 0; e < r; ++e)
        dot += ora_load(pool, elem_bytes, (size_t)a * r + e) * ora_load(pool, elem_bytes, (size_t)b * r + e);
    return dot / (norm[a] * norm[b]);
}

/* Dense similarity of a node: S[i*mr + j] = cos(K[L[i]], K[R[j]]). */
void ora_similarity(const void *kpool, int elem_bytes, int r, const double *norm_k,
                    const int32_t *L, int ml, const int32_t *R, int mr, double *S)
{
    for (int i = 0; i < ml; ++i)
        for (int j = 0; j < mr; ++j)
            S[(size_t)i * mr + j] = ora_cosine(kpool, elem_bytes, r, norm_k, L[i], R[j]);
}

/* Threshold line of Algorithm 1 under the one-target reading: for right block
 * j the candidate row is the smallest i attaining max_i S[i][j]; it is fused
 * iff that maximum is > thr.  assign[j] = i or -1.  best[j], second[j] = the
 * largest and second largest value in column j (second = -inf if ml < 2);
 * both may be NULL. */
void ora_assign(const double *S, int ml, int mr, double thr, int32_t *assign, double *best, double *second)
{
    for (int j = 0; j < mr; ++j) {
        double b = -INFINITY, s2 = -INFINITY;
        int bi = -1;
        for (int i = 0; i < ml; ++i) {
            double s = S[(size_t)i * mr + j];
            if (s > b) {
                s2 = b;
                b = s;
                bi = i;
            } else if (s > s2) {
                s2 = s;
            }
        }
        assign[j] = (bi >= 0 && b > thr) ? bi : -1;
        if (best)
            best[j] = b;
        if (second)
            second[j] = s2;
    }
}

/* Threshold line of Algorithm 1 under the row-order reading (the loop over
 * the rows of sim, taken literally): rows are visited in ascending order; a
 * row takes every right block whose cosine with it is > thr and that no
 * earlier row has taken, and a taken block is evicted at once, so later rows
 * no longer see it.  assign[j] = the row that took j, or -1. */
void ora_assign_first_row(const double *S, int ml, int mr, double thr, int32_t *assign)
{
    for (int j = 0; j < mr; ++j)
        assign[j] = -1;
    for (int i = 0; i < ml; ++i)
        for (int j = 0; j < mr; ++j) {
            if (assign[j] >= 0)
                continue; /* evicted by an earlier row */
            if (S[(size_t)i * mr + j] > thr)
                assign[j] = i;
        }
}

/* Fusion lines of Algorithm 1 for one pool tensor (call once for K, once for
 * V with the same assign[]): for every left row i with at least one fused
 * right block, stored(L[i]) <- round(normalize(u(L[i]) + sum_j u(R[j]))),
 * members j in ascending order, u(x) = x/||x||; then norm[L[i]] is recomputed
 * from the rounded values.  Rows of R are only read. */
void ora_merge(void *pool, int elem_bytes, int r, double *norm,
               const int32_t *L, int ml, const int32_t *R, int mr, const int32_t *assign)
{
    double *acc = (double *)malloc(sizeof(double) * (size_t)r);
    for (int i = 0; i < ml; ++i) {
        int any = 0;
        for (int j = 0; j < mr; ++j)
            if (assign[j] == i)
                any = 1;
        if (!any)
            continue;
        int a = L[i];
        for (int e = 0; e < r; ++e)
            acc[e] = (norm[a] == 0.0) ? 0.0 : ora_load(pool, elem_bytes, (size_t)a * r + e) / norm[a];
        for (int j = 0; j < mr; ++j) {
            if (assign[j] != i)
                continue;
            int b = R[j];
            if (norm[b] == 0.0)
                continue;
            for (int e = 0; e < r; ++e)
                acc[e] += ora_load(pool, elem_bytes, (size_t)b * r + e) / norm[b];
        }
        double ss = 0.0;
        for (int e = 0; e < r; ++e)
            ss += acc[e] * acc[e];
        double len = sqrt(ss);
        double ss_stored = 0.0;
        for (int e = 0; e < r; ++e) {
            double u = (len == 0.0) ? 0.0 : acc[e] / len;
            ora_store(pool, elem_bytes, (size_t)a * r + e, u);
            double back = ora_load(pool, elem_bytes, (size_t)a * r + e);
            ss_stored += back * back;
        }
        norm[a] = sqrt(ss_stored);
    }
    free(acc);
}

/* "evict fused blocks", "update block-table": repoint logical blocks, add up
 * reference counts, append evicted ids to the free list (in eviction order),
 * and refresh the scale of EVERY logical block that points at a rewritten
 * left row.  bt, scale_*, refcount are in/out. */
void ora_rewrite(int32_t *bt, int n, const int32_t *L, int ml, const int32_t *R, int mr,
                 const int32_t *assign, const double *orig_norm_k, const double *orig_norm_v,
                 const double *norm_k, const double *norm_v, double *scale_k, double *scale_v,
                 int32_t *refcount, int32_t *free_list, int32_t *n_free)
{
    (void)ml;
    for (int j = 0; j < mr; ++j) {
        if (assign[j] < 0)
            continue;
        int from = R[j], to = L[assign[j]];
        for (int x = 0; x < n; ++x)
            if (bt[x] == from)
                bt[x] = to;
        refcount[to] += refcount[from];
        refcount[from] = 0;
        free_list[(*n_free)++] = from;
    }
    for (int j = 0; j < mr; ++j) {
        if (assign[j] < 0)
            continue;
        int to = L[assign[j]];
        for (int x = 0; x < n; ++x) {
            if (bt[x] != to)
                continue;
            scale_k[x] = (norm_k[to] == 0.0) ? 0.0 : orig_norm_k[x] / norm_k[to];
            scale_v[x] = (norm_v[to] == 0.0) ? 0.0 : orig_norm_v[x] / norm_v[to];
        }
    }
}

/* ------------------------------------------------------------------ */
/* Algorithm 1: the recursion                                          */
/* ------------------------------------------------------------------ */

/* Host threads that share out the columns of one node (1 = none).  Set once before a run; it changes how long a run
 * takes and nothing that it computes. */
static int ora_column_threads = 1;
void ora_set_column_threads(int n) { ora_column_threads = n > 1 ? n : 1; }

typedef struct {
    int elem_bytes, r, P, n;
    void *kpool, *vpool;
    int32_t *bt;
    const int32_t *leaf_start, *leaf_count;
    double thr, band;
    int rule; /* 0: one target per right block by arg-max; 1: row order, the first row above thr takes the block */
    double *orig_norm_k, *orig_norm_v, *norm_k, *norm_v, *scale_k, *scale_v;
    int32_t *refcount, *free_list, *n_free;
    /* decision statistics */
    int64_t n_decisions, n_fused, n_near_thr, n_exact_tie;
    double min_thr_margin, min_tie_gap;
    /* optional trace of every decision: (right phys id, target phys id or -1) */
    int32_t *trace;
    int64_t trace_cap, trace_len;
} ora_ctx;

typedef struct {
    int32_t *id;
    int m;
} ora_set;

/* One internal node: fuse the right set into the left set, return the
 * concatenation of the left set and the non-fused right blocks. */
static ora_set ora_node(ora_ctx *c, ora_set Ls, ora_set Rs)
{
    int ml = Ls.m, mr = Rs.m;
    int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * (size_t)(mr > 0 ? mr : 1));
    double *best_of = (double *)malloc(sizeof(double) * (size_t)(mr > 0 ? mr : 1));
    double *second_of = (double *)malloc(sizeof(double) * (size_t)(mr > 0 ? mr : 1));
    /* Column by column so that the dense matrix need not be held.  The columns of a node are independent (sim is
     * computed once, before any fusing), so they may be shared out over host threads; every cosine is still one
     * left-to-right fp64 sum and every decision is taken on its own column, whatever the thread count. */
#pragma omp parallel num_threads(ora_column_threads) if (ora_column_threads > 1 && mr > 1)
    {
        double *col = (double *)malloc(sizeof(double) * (size_t)(ml > 0 ? ml : 1));
#pragma omp for schedule(dynamic, 8)
        for (int j = 0; j < mr; ++j) {
            for (int i = 0; i < ml; ++i)
                col[i] = ora_cosine(c->kpool, c->elem_bytes, c->r, c->norm_k, Ls.id[i], Rs.id[j]);
            double best, second;
            ora_assign(col, ml, 1, c->thr, &assign[j], &best, &second);
            if (c->rule == 1) {
                /* the column seen by the row loop; the value that decided it is the taker's cosine, or the column
                 * maximum when no row took it */
                ora_assign_first_row(col, ml, 1, c->thr, &assign[j]);
                if (assign[j] >= 0)
                    best = col[assign[j]];
            }
            best_of[j] = best;
            second_of[j] = second;
        }
        free(col);
    }
    /* statistics and the optional trace, in column order; they never feed back into a decision */
    for (int j = 0; j < mr; ++j) {
        double best = best_of[j], second = second_of[j];
        if (ml > 0) {
            c->n_decisions++;
            double mg = fabs(best - c->thr);
            if (mg < c->min_thr_margin)
                c->min_thr_margin = mg;
            if (mg <= c->band)
                c->n_near_thr++;
            if (assign[j] >= 0) {
                c->n_fused++;
                if (c->rule == 1)
                    ; /* ties between rows play no part in the row-order reading */
                else if (best == second)
                    c->n_exact_tie++;
                else if (best - second < c->min_tie_gap)
                    c->min_tie_gap = best - second;
            }
        }
        if (c->trace && c->trace_len + 2 <= c->trace_cap) {
            c->trace[c->trace_len++] = Rs.id[j];
            c->trace[c->trace_len++] = assign[j] >= 0 ? Ls.id[assign[j]] : -1;
        }
    }
    free(best_of);
    free(second_of);
    ora_merge(c->kpool, c->elem_bytes, c->r, c->norm_k, Ls.id, ml, Rs.id, mr, assign);
    ora_merge(c->vpool, c->elem_bytes, c->r, c->norm_v, Ls.id, ml, Rs.id, mr, assign);
    ora_rewrite(c->bt, c->n, Ls.id, ml, Rs.id, mr, assign, c->orig_norm_k, c->orig_norm_v,
                c->norm_k, c->norm_v, c->scale_k, c->scale_v, c->refcount, c->free_list, c->n_free);
    ora_set out;
    out.id = (int32_t *)malloc(sizeof(int32_t) * (size_t)(ml + mr > 0 ? ml + mr : 1));
    out.m = 0;
    for (int i = 0; i < ml; ++i)
        out.id[out.m++] = Ls.id[i];
    for (int j = 0; j < mr; ++j)
        if (assign[j] < 0)
            out.id[out.m++] = Rs.id[j];
    free(assign);
    free(Ls.id);
    free(Rs.id);
    return out;
}

/* FastFusion over leaves [lo, hi): split at len//2, left first. */
static ora_set ora_ff_leaves(ora_ctx *c, int lo, int hi)
{
    if (hi - lo == 1) {
        ora_set s;
        s.m = c->leaf_count[lo];
        s.id = (int32_t *)malloc(sizeof(int32_t) * (size_t)(s.m > 0 ? s.m : 1));
        for (int x = 0; x < s.m; ++x)
            s.id[x] = c->bt[c->leaf_start[lo] + x];
        return s;
    }
    int mid = lo + (hi - lo) / 2;
    ora_set L = ora_ff_leaves(c, lo, mid);
    ora_set R = ora_ff_leaves(c, mid, hi);
    return ora_node(c, L, R);
}

/* FastFusion over units (requests) [lo, hi); a unit with several leaves
 * (chunks) is first fused over its own leaves. */
static ora_set ora_ff_units(ora_ctx *c, const int32_t *unit_leaf_ptr, int lo, int hi)
{
    if (hi - lo == 1) {
        if (unit_leaf_ptr[lo + 1] == unit_leaf_ptr[lo]) {
            ora_set s;
            s.m = 0;
            s.id = (int32_t *)malloc(sizeof(int32_t));
            return s;
        }
        return ora_ff_leaves(c, unit_leaf_ptr[lo], unit_leaf_ptr[lo + 1]);
    }
    int mid = lo + (hi - lo) / 2;
    ora_set L = ora_ff_units(c, unit_leaf_ptr, lo, mid);
    ora_set R = ora_ff_units(c, unit_leaf_ptr, mid, hi);
    return ora_node(c, L, R);
}

/*
 * Whole pipeline for one group.
 *
 *   kpool, vpool  [P][r] storage type, modified in place (fused rows only)
 *   bt            [n] logical -> physical, in/out; must be injective on entry
 *   leaves        leaf l = logical entries leaf_start[l] .. +leaf_count[l]
 *   units         unit u = leaves unit_leaf_ptr[u] .. unit_leaf_ptr[u+1]
 *   group_size    the method's "every N requests or chunks": consecutive runs
 *                 of N units (or, when there is one unit, N leaves) form
 *                 independent trees; <= 0 means one tree over everything
 *   outputs       orig_norm_* [n], norm_* [P], scale_* [n], refcount [P],
 *                 free_list [P] + *n_free, stats[8], optional trace
 *   rule          0 = arg-max reading of the threshold line, 1 = row-order reading
 * stats: 0 decisions, 1 fused, 2 near-threshold (|best-thr| <= band),
 *        3 exact ties among fused, 4 min |best-thr|, 5 min positive tie gap,
 *        6 distinct physical blocks after fusion, 7 compression ratio n/distinct
 */
int ora_fuse_group(int elem_bytes, int r, int P, int n, void *kpool, void *vpool, int32_t *bt,
                   const int32_t *leaf_start, const int32_t *leaf_count, int n_leaves,
                   const int32_t *unit_leaf_ptr, int n_units, int group_size, double thr, double band,
                   double *orig_norm_k, double *orig_norm_v, double *norm_k, double *norm_v,
                   double *scale_k, double *scale_v, int32_t *refcount, int32_t *free_list,
                   int32_t *n_free, double *stats, int32_t *trace, int64_t trace_cap, int64_t *trace_len, int rule)
{
    if ((elem_bytes != 2 && elem_bytes != 4) || r <= 0 || P <= 0 || n < 0)
        return -1;
    ora_ctx c;
    memset(&c, 0, sizeof(c));
    c.elem_bytes = elem_bytes; c.r = r; c.P = P; c.n = n;
    c.kpool = kpool; c.vpool = vpool; c.bt = bt;
    c.leaf_start = leaf_start; c.leaf_count = leaf_count;
    c.thr = thr; c.band = band; c.rule = rule;
    c.orig_norm_k = orig_norm_k; c.orig_norm_v = orig_norm_v;
    c.norm_k = norm_k; c.norm_v = norm_v; c.scale_k = scale_k; c.scale_v = scale_v;
    c.refcount = refcount; c.free_list = free_list; c.n_free = n_free;
    c.min_thr_margin = INFINITY; c.min_tie_gap = INFINITY;
    c.trace = trace; c.trace_cap = trace_cap; c.trace_len = 0;
    *n_free = 0;

    /* leaf step: store norms, identity scales, one reference per used block */
    ora_block_norms(kpool, elem_bytes, r, P, norm_k);
    ora_block_norms(vpool, elem_bytes, r, P, norm_v);
    for (int b = 0; b < P; ++b)
        refcount[b] = 0;
    for (int x = 0; x < n; ++x) {
        if (bt[x] < 0 || bt[x] >= P)
            return -2;
        orig_norm_k[x] = norm_k[bt[x]];
        orig_norm_v[x] = norm_v[bt[x]];
        scale_k[x] = 1.0;
        scale_v[x] = 1.0;
        if (refcount[bt[x]] != 0)
            return -3; /* table must be injective before fusion */
        refcount[bt[x]] = 1;
    }

    if (n_units == 1) {
        int lo = unit_leaf_ptr[0], hi = unit_leaf_ptr[1];
        int step = group_size > 0 ? group_size : (hi - lo > 0 ? hi - lo : 1);
        for (int a = lo; a < hi; a += step) {
            int b = a + step < hi ? a + step : hi;
            ora_set s = ora_ff_leaves(&c, a, b);
            free(s.id);
        }
    } else {
        int step = group_size > 0 ? group_size : (n_units > 0 ? n_units : 1);
        for (int a = 0; a < n_units; a += step) {
            int b = a + step < n_units ? a + step : n_units;
            ora_set s = ora_ff_units(&c, unit_leaf_ptr, a, b);
            free(s.id);
        }
    }
    (void)n_leaves;

    int distinct = 0;
    for (int b = 0; b < P; ++b)
        if (refcount[b] > 0)
            distinct++;
    stats[0] = (double)c.n_decisions; stats[1] = (double)c.n_fused;
    stats[2] = (double)c.n_near_thr;  stats[3] = (double)c.n_exact_tie;
    stats[4] = c.min_thr_margin;      stats[5] = c.min_tie_gap;
    stats[6] = (double)distinct;
    stats[7] = distinct > 0 ? (double)n / (double)distinct : 0.0; /* compression ratio = logical / physical */
    if (trace_len)
        *trace_len = c.trace_len;
    return 0;
}
