/* Drives the CPU oracle (oracle/octfd_oracle.c) through every exported pipeline call on a small three-level
 * tree.  tests/test_sanitizers.py builds the two files together with gcc -fsanitize=address,undefined
 * -fno-sanitize-recover=all: an out-of-bounds access, a leak or an undefined operation anywhere in the oracle
 * ends the run with a report.  Values are only required to be finite here; what they must equal is the
 * business of the pin tests. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t orc_tree_build(int lmin, int lmax, int npts, const uint32_t *pts, const uint32_t *radius, void **out);
int64_t orc_tree_from_leaves(const uint32_t *lv, int64_t n, void **out);
void orc_tree_leaves(const void *t, uint32_t *out);
void orc_tree_free(void *t);
int orc_ghost_table(const void *t, int32_t *out);
void orc_unzip(const void *t, int nvar, const double *zipped, double *padded, const int64_t *blocks, int64_t nsel);
void orc_unzip_centred(const void *t, int nvar, const double *zipped, double *padded);
void orc_F(const void *t, int kind, double sigma, const double *zipped, const int64_t *blocks, int64_t nsel, double *out);
int orc_rk4_step(const void *t, int kind, double sigma, double dt, double *u);
int orc_rk4_step_centred(const void *t, int kind, double sigma, double dt, double *u);
int orc_transfer(const void *src, const void *dst, int nvar, const double *in, double *out);

static int finite_all(const double *v, size_t n)
{
    for (size_t i = 0; i < n; i++) if (!isfinite(v[i])) return 0;
    return 1;
}

int main(void)
{
    int failures = 0;
    uint32_t pa[6] = {500000, 520000, 540000, 300000, 700000, 410000}, pb[6] = {520000, 520000, 540000, 300000, 690000, 410000};
    uint32_t rad[2] = {60000, 40000}, huge[2] = {0xffffffffu, 1};
    void *ta = NULL, *tb = NULL, *tc = NULL;
    int64_t na = orc_tree_build(3, 5, 2, pa, rad, &ta), nb = orc_tree_build(3, 5, 2, pb, rad, &tb);
    printf("trees of %ld and %ld blocks\n", (long)na, (long)nb);
    if (na <= 512 || nb <= 512) { printf("FAILED: tree build\n"); return 1; }
    if (orc_tree_build(3, 5, 2, pa, huge, &tc) >= 0) { printf("FAILED: a radius beyond 2^21 was accepted\n"); failures++; }
    int32_t *gt = malloc((size_t)na * 27 * 5 * sizeof(int32_t));
    if (orc_ghost_table(ta, gt)) { printf("FAILED: ghost table\n"); failures++; }
    free(gt);
    /* the same tree from its own leaf list */
    uint32_t *lv = malloc((size_t)na * 4 * sizeof(uint32_t));
    orc_tree_leaves(ta, lv);
    void *td = NULL;
    if (orc_tree_from_leaves(lv, na, &td) != na) { printf("FAILED: from leaves\n"); failures++; }
    orc_tree_free(td);
    td = NULL;
    if (orc_tree_from_leaves(lv, na - 1, &td) >= 0) { printf("FAILED: a missing leaf was accepted\n"); failures++; }
    orc_tree_free(td);
    free(lv);
    /* fields: smooth and bounded */
    const size_t BLK = 512, PBLK = 2744;
    double *u = malloc(24 * (size_t)na * BLK * sizeof(double)), *k = malloc(24 * (size_t)na * BLK * sizeof(double));
    for (size_t i = 0; i < 24 * (size_t)na * BLK; i++) u[i] = 0.3 * sin(0.001 * (double)i) + 0.1 * cos(0.37 * (double)(i % 977));
    double *pad = malloc(2 * (size_t)na * PBLK * sizeof(double));
    orc_unzip(ta, 2, u, pad, NULL, na);
    failures += !finite_all(pad, 2 * (size_t)na * PBLK);
    orc_unzip_centred(ta, 2, u, pad);
    failures += !finite_all(pad, 2 * (size_t)na * PBLK);
    free(pad);
    for (int kind = 0; kind < 4; kind++) {
        orc_F(ta, kind, 0.4, u, NULL, na, k);
        const int nvo = kind == 0 ? 4 : (kind == 1 ? 2 : (kind == 2 ? 1 : 24));
        if (!finite_all(k, (size_t)nvo * na * BLK)) { printf("FAILED: F of kind %d\n", kind); failures++; }
    }
    int64_t some[3] = {0, na / 2, na - 1};
    orc_F(ta, 3, 0.4, u, some, 3, k);
    failures += !finite_all(k, 24 * 3 * BLK);
    for (int kind = 1; kind < 4; kind++) {
        if (orc_rk4_step(ta, kind, 0.4, ldexp(1.0, -10), u)) { printf("FAILED: rk4 of kind %d\n", kind); failures++; }
        if (kind < 3 && orc_rk4_step_centred(ta, kind, 0.4, ldexp(1.0, -10), u)) { printf("FAILED: centred rk4 of kind %d\n", kind); failures++; }
    }
    if (orc_rk4_step(ta, 0, 0.0, 1e-3, u) == 0) { printf("FAILED: rk4 of a kind that cannot be stepped\n"); failures++; }
    double *v = malloc(2 * (size_t)nb * BLK * sizeof(double));
    if (orc_transfer(ta, tb, 2, u, v)) { printf("FAILED: transfer\n"); failures++; }
    failures += !finite_all(v, 2 * (size_t)nb * BLK);
    free(v); free(u); free(k);
    orc_tree_free(ta); orc_tree_free(tb); orc_tree_free(tc);
    printf(failures ? "FAILED\n" : "all oracle calls ran clean\n");
    return failures ? 1 : 0;
}
