/*
 * Runs ora_fuse_group of the CPU oracle on a problem read from a file, for builds of the oracle under the address and
 * undefined-behaviour sanitizers.  TEST INFRASTRUCTURE ONLY, like the oracle itself: tests/test_sanitizers.py
 * compiles this file together with kvfuse_oracle.c, runs it on a small seeded problem and compares what it writes
 * with the ordinary build of the oracle.  No arithmetic of its own.
 *
 * Input file:  int32 header {elem_bytes, r, P, n, n_leaves, n_units, group_size, rule}, double {thr, band},
 *              kpool [P*r*elem_bytes], vpool (same), bt int32 [n], leaf_start, leaf_count int32 [n_leaves],
 *              unit_leaf_ptr int32 [n_units + 1].
 * Output file: bt int32 [n], refcount int32 [P], kpool, vpool (as read), scale_k, scale_v double [n], stats double [8].
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "kvfuse_oracle.c"

static void *rd(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) {
        fprintf(stderr, "sanitize_driver: short read\n");
        exit(2);
    }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s input output\n", argv[0]);
        return 2;
    }
    FILE *f = fopen(argv[1], "rb");
    if (!f)
        return 2;
    int32_t *h = (int32_t *)rd(f, 8 * sizeof(int32_t));
    double *t = (double *)rd(f, 2 * sizeof(double));
    const int eb = h[0], r = h[1], P = h[2], n = h[3], nl = h[4], nu = h[5], gs = h[6], rule = h[7];
    const size_t pool_bytes = (size_t)P * (size_t)r * (size_t)eb;
    void *kpool = rd(f, pool_bytes), *vpool = rd(f, pool_bytes);
    int32_t *bt = (int32_t *)rd(f, sizeof(int32_t) * (size_t)n);
    int32_t *ls = (int32_t *)rd(f, sizeof(int32_t) * (size_t)nl), *lc = (int32_t *)rd(f, sizeof(int32_t) * (size_t)nl);
    int32_t *up = (int32_t *)rd(f, sizeof(int32_t) * (size_t)(nu + 1));
    fclose(f);
    double *onk = calloc((size_t)n + 1, sizeof(double)), *onv = calloc((size_t)n + 1, sizeof(double));
    double *nk = calloc((size_t)P, sizeof(double)), *nv = calloc((size_t)P, sizeof(double));
    double *sk = calloc((size_t)n + 1, sizeof(double)), *sv = calloc((size_t)n + 1, sizeof(double));
    int32_t *rc = calloc((size_t)P, sizeof(int32_t)), *fl = calloc((size_t)P, sizeof(int32_t));
    int32_t n_free = 0;
    double stats[8];
    int64_t trace_len = 0;
    ora_set_column_threads(2);
    const int ret = ora_fuse_group(eb, r, P, n, kpool, vpool, bt, ls, lc, nl, up, nu, gs, t[0], t[1], onk, onv, nk, nv, sk, sv, rc,
                                   fl, &n_free, stats, NULL, 0, &trace_len, rule);
    if (ret != 0)
        return 3;
    FILE *o = fopen(argv[2], "wb");
    if (!o)
        return 2;
    fwrite(bt, sizeof(int32_t), (size_t)n, o);
    fwrite(rc, sizeof(int32_t), (size_t)P, o);
    fwrite(kpool, 1, pool_bytes, o);
    fwrite(vpool, 1, pool_bytes, o);
    fwrite(sk, sizeof(double), (size_t)n, o);
    fwrite(sv, sizeof(double), (size_t)n, o);
    fwrite(stats, sizeof(double), 8, o);
    fclose(o);
    free(h); free(t); free(kpool); free(vpool); free(bt); free(ls); free(lc); free(up);
    free(onk); free(onv); free(nk); free(nv); free(sk); free(sv); free(rc); free(fl);
    return 0;
}
