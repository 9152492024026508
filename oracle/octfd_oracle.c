/*
 * octfd_oracle.c -- plain CPU reference ("oracle") for the block finite-difference pipeline
 * on a 2:1-balanced, periodic, Morton-ordered octree of 8^3-point blocks.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library and to be timed as a
 * CPU baseline.  Only the tests, the smoke check and the benchmark's cpu-baseline leg may
 * load it; the product library never calls it and shares no code with it.
 *
 * The source paper (a data-parallel deep-learning framework for a neural Burgers solver)
 * gives exactly one governing equation, the inviscid Burgers equation u_t + u u_x = 0 of its
 * introduction (Eq. "Inviscid_Burgers"); it is silent on octrees, ghost padding, stencil
 * order, dissipation and time integration.  Every definition below is therefore the textbook
 * one, written out slowly:
 *
 *   lattice     level-l lattice has N_l = 8*2^l points per axis, spacing h_l = 2^-(l+3),
 *               periodic; point I of level l is point 2I of level l+1 (vertex aligned).
 *   leaf/block  leaf (l,a) owns points I = 8a+i, i=0..7 per axis.
 *   build       refine an octant of level l<lmax when a seed point is closer than R_l to its
 *               closed box (integers on the 2^20 lattice, periodic images); then enforce the
 *               26-neighbour 2:1 balance to its (unique) minimal fixed point; sort by Morton key.
 *   unzip       every one of the 14^3 points of a padded block takes the value of the leaf
 *               that contains it: copy (same level), injection (finer leaf), or 6-point
 *               Lagrange interpolation from the 8 stored nodes of a coarser leaf (x, then y,
 *               then z; even fine coordinates pass through).
 *   stencils    6th-order centred first/second derivatives, mixed second derivatives as
 *               D1_a(D1_b u), 6th-difference Kreiss-Oliger dissipation.
 *   rhs kinds   DERIVS, WAVE, BURGERS (the paper's equation), SYN24 (24-field synthetic system).
 *   rk4         classical four-stage Runge-Kutta on zipped vectors.
 *   transfer    after a regrid, every point of the new tree takes the old tree's value there:
 *               copy, injection, or the same Lagrange interpolation from a one-level-coarser leaf.
 *
 * Floating point: fp64, one fixed IEEE operation sequence per formula (explicit fma() where a
 * fused multiply-add is meant; compile with -ffp-contract=off so nothing else is fused).
 * No blocking, tiling or table-driven indexing: ghost values are found by point location.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NPT 8   /* owned points per axis per block */
#define PAD 3   /* ghost layers                     */
#define NP (NPT + 2 * PAD) /* 14 */
#define BLK (NPT * NPT * NPT)  /* 512  */
#define PBLK (NP * NP * NP)    /* 2744 */
#define QBITS 20               /* seed points and radii live on the 2^20 lattice */
#define MAXLEVEL 19

enum { ORC_DERIVS = 0, ORC_WAVE = 1, ORC_BURGERS = 2, ORC_SYN24 = 3 };
enum { G_SAME = 0, G_FINER = 1, G_COARSER = 2 };

typedef struct { uint32_t level, ix, iy, iz; } orc_leaf;

typedef struct {
    int64_t n;          /* number of live leaves after finalisation          */
    int64_t cap, used;  /* dynamic leaf array during construction            */
    orc_leaf *leaves;
    uint8_t *alive;     /* construction only                                  */
    /* open-addressing hash  key(l,ix,iy,iz) -> index into leaves            */
    uint64_t hcap, hcount;
    uint64_t *hkey;
    int64_t *hval;      /* -1 = removed (split)                               */
} orc_tree;

/* ------------------------------------------------------------------ hash of octants */

static uint64_t okey(uint32_t l, uint32_t ix, uint32_t iy, uint32_t iz)
{
    return ((uint64_t)l << 57) | ((uint64_t)iz << 38) | ((uint64_t)iy << 19) | (uint64_t)ix;
}
#define EMPTY_KEY UINT64_MAX

static uint64_t mix64(uint64_t z)
{
    z ^= z >> 33; z *= 0xff51afd7ed558ccdULL; z ^= z >> 33; z *= 0xc4ceb9fe1a85ec53ULL; z ^= z >> 33;
    return z;
}

static void hash_alloc(orc_tree *t, uint64_t cap)
{
    t->hcap = cap; t->hcount = 0;
    t->hkey = (uint64_t *)malloc(cap * sizeof(uint64_t));
    t->hval = (int64_t *)malloc(cap * sizeof(int64_t));
    for (uint64_t i = 0; i < cap; i++) t->hkey[i] = EMPTY_KEY;
}

static void hash_put(orc_tree *t, uint64_t key, int64_t val);

static void hash_grow(orc_tree *t)
{
    uint64_t ocap = t->hcap; uint64_t *ok = t->hkey; int64_t *ov = t->hval;
    hash_alloc(t, ocap * 2);
    for (uint64_t i = 0; i < ocap; i++) if (ok[i] != EMPTY_KEY) hash_put(t, ok[i], ov[i]);
    free(ok); free(ov);
}

static void hash_put(orc_tree *t, uint64_t key, int64_t val)
{
    if (2 * (t->hcount + 1) > t->hcap) hash_grow(t);
    uint64_t m = t->hcap - 1, p = mix64(key) & m;
    while (t->hkey[p] != EMPTY_KEY && t->hkey[p] != key) p = (p + 1) & m;
    if (t->hkey[p] == EMPTY_KEY) { t->hkey[p] = key; t->hcount++; }
    t->hval[p] = val;
}

/* index of the live leaf with this exact key, or -1 */
static int64_t hash_get(const orc_tree *t, uint64_t key)
{
    uint64_t m = t->hcap - 1, p = mix64(key) & m;
    while (t->hkey[p] != EMPTY_KEY) {
        if (t->hkey[p] == key) return t->hval[p];
        p = (p + 1) & m;
    }
    return -1;
}

/* ------------------------------------------------------------------ construction */

static int64_t leaf_append(orc_tree *t, uint32_t l, uint32_t ix, uint32_t iy, uint32_t iz)
{
    if (t->used == t->cap) {
        t->cap *= 2;
        t->leaves = (orc_leaf *)realloc(t->leaves, t->cap * sizeof(orc_leaf));
        t->alive = (uint8_t *)realloc(t->alive, t->cap);
    }
    int64_t i = t->used++;
    t->leaves[i].level = l; t->leaves[i].ix = ix; t->leaves[i].iy = iy; t->leaves[i].iz = iz;
    t->alive[i] = 1;
    hash_put(t, okey(l, ix, iy, iz), i);
    return i;
}

static void leaf_split(orc_tree *t, int64_t i)
{
    orc_leaf p = t->leaves[i];
    t->alive[i] = 0;
    hash_put(t, okey(p.level, p.ix, p.iy, p.iz), -1);
    for (uint32_t c = 0; c < 8; c++)
        leaf_append(t, p.level + 1, 2 * p.ix + (c & 1), 2 * p.iy + ((c >> 1) & 1), 2 * p.iz + ((c >> 2) & 1));
}

/* squared distance (2^20-lattice units) from seed point c to the closed box of octant (l,a),
 * minimum over the three periodic images of the point per axis */
static int64_t axis_gap(int64_t c, int64_t lo, int64_t hi)
{
    int64_t best = INT64_MAX;
    for (int im = -1; im <= 1; im++) {
        int64_t cc = c + (int64_t)im * ((int64_t)1 << QBITS);
        int64_t g = cc < lo ? lo - cc : (cc > hi ? cc - hi : 0);
        if (g < best) best = g;
    }
    return best;
}

static int wants_refine(const orc_leaf *o, int lmin, int lmax, int npts, const uint32_t *pts, const uint32_t *radius)
{
    if ((int)o->level >= lmax) return 0;
    int64_t s = (int64_t)1 << (QBITS - o->level);
    int64_t R = radius[o->level - lmin];
    const uint32_t a[3] = { o->ix, o->iy, o->iz };
    for (int p = 0; p < npts; p++) {
        int64_t d2 = 0;
        for (int d = 0; d < 3; d++) {
            int64_t g = axis_gap(pts[3 * p + d], a[d] * s, (a[d] + 1) * s);
            d2 += g * g;
        }
        if (d2 < R * R) return 1;
    }
    return 0;
}

/* live leaf that contains octant (l,a), searching l, l-1, ..., 0; -1 if the octant is subdivided */
static int64_t container_of_octant(const orc_tree *t, uint32_t l, uint32_t ix, uint32_t iy, uint32_t iz)
{
    for (int ll = (int)l; ll >= 0; ll--) {
        int sh = (int)l - ll;
        int64_t i = hash_get(t, okey(ll, ix >> sh, iy >> sh, iz >> sh));
        if (i >= 0) return i;
    }
    return -1;
}

static uint64_t morton_key(const orc_leaf *o)
{
    int sh = QBITS - (int)o->level;
    uint64_t x = (uint64_t)o->ix << sh, y = (uint64_t)o->iy << sh, z = (uint64_t)o->iz << sh, k = 0;
    for (int b = 0; b < QBITS; b++)
        k |= ((x >> b) & 1) << (3 * b) | ((y >> b) & 1) << (3 * b + 1) | ((z >> b) & 1) << (3 * b + 2);
    return k;
}

static int cmp_leaf(const void *pa, const void *pb)
{
    uint64_t a = morton_key((const orc_leaf *)pa), b = morton_key((const orc_leaf *)pb);
    return a < b ? -1 : (a > b ? 1 : 0);
}

static orc_tree *tree_new(void)
{
    orc_tree *t = (orc_tree *)calloc(1, sizeof(orc_tree));
    t->cap = 1024; t->used = 0;
    t->leaves = (orc_leaf *)malloc(t->cap * sizeof(orc_leaf));
    t->alive = (uint8_t *)malloc(t->cap);
    hash_alloc(t, 4096);
    return t;
}

/* compact the live leaves, sort by Morton key, rebuild the hash onto final indices */
static void tree_finalise(orc_tree *t)
{
    int64_t n = 0;
    for (int64_t i = 0; i < t->used; i++) if (t->alive[i]) t->leaves[n++] = t->leaves[i];
    t->n = n; t->used = n;
    qsort(t->leaves, (size_t)n, sizeof(orc_leaf), cmp_leaf);
    free(t->hkey); free(t->hval);
    uint64_t cap = 4096; while (cap < (uint64_t)(4 * n)) cap *= 2;
    hash_alloc(t, cap);
    for (int64_t i = 0; i < n; i++) {
        t->alive[i] = 1;
        hash_put(t, okey(t->leaves[i].level, t->leaves[i].ix, t->leaves[i].iy, t->leaves[i].iz), i);
    }
}

/* 26-neighbour periodic 2:1 balance, swept to a fixed point.  Returns number of splits. */
static int64_t balance(orc_tree *t)
{
    int64_t splits = 0; int changed = 1;
    while (changed) {
        changed = 0;
        for (int64_t i = 0; i < t->used; i++) {           /* t->used grows while we sweep */
            if (!t->alive[i]) continue;
            orc_leaf o = t->leaves[i];
            if (o.level == 0) continue;
            uint32_t m = (1u << o.level) - 1;
            for (int dz = -1; dz <= 1; dz++) for (int dy = -1; dy <= 1; dy++) for (int dx = -1; dx <= 1; dx++) {
                if (!dx && !dy && !dz) continue;
                uint32_t nx = (o.ix + (uint32_t)dx) & m, ny = (o.iy + (uint32_t)dy) & m, nz = (o.iz + (uint32_t)dz) & m;
                for (;;) {
                    int64_t c = container_of_octant(t, o.level, nx, ny, nz);
                    if (c < 0 || t->leaves[c].level + 1 >= o.level) break;
                    leaf_split(t, c); splits++; changed = 1;
                }
            }
        }
    }
    return splits;
}

/* Build: uniform lmin, predicate refinement, balance, sort.  Returns leaf count (<0 on bad args). */
int64_t orc_tree_build(int lmin, int lmax, int npts, const uint32_t *pts, const uint32_t *radius, void **out)
{
    if (lmin < 3 || lmax < lmin || lmax > MAXLEVEL || npts < 0 || !out) return -1;
    for (int l = lmin; l < lmax; l++)                     /* radii beyond twice the cube's edge: rejected (R*R stays far from 2^63) */
        if (radius[l - lmin] > (2u << QBITS)) return -1;
    orc_tree *t = tree_new();
    uint32_t n0 = 1u << lmin;
    for (uint32_t z = 0; z < n0; z++) for (uint32_t y = 0; y < n0; y++) for (uint32_t x = 0; x < n0; x++)
        leaf_append(t, (uint32_t)lmin, x, y, z);
    for (int64_t i = 0; i < t->used; i++) {               /* children are appended and visited later */
        if (!t->alive[i]) continue;
        orc_leaf o = t->leaves[i];
        if (wants_refine(&o, lmin, lmax, npts, pts, radius)) leaf_split(t, i);
    }
    balance(t);
    tree_finalise(t);
    *out = t;
    return t->n;
}

/* Tree from an explicit leaf list (any order).  Returns n, or -3 if not 26-balanced,
 * -4 if the leaves do not tile the cube exactly once. */
int64_t orc_tree_from_leaves(const uint32_t *lv, int64_t n, void **out)
{
    orc_tree *t = tree_new();
    /* exact volume check in units of 8^-MAXLEVEL would overflow; use long double sum of 8^-l and
     * pairwise non-containment through the hash instead */
    long double vol = 0.0L;
    for (int64_t i = 0; i < n; i++) {
        uint32_t l = lv[4 * i];
        if (l > MAXLEVEL || lv[4 * i + 1] >> l || lv[4 * i + 2] >> l || lv[4 * i + 3] >> l) { *out = t; return -1; }
        if (hash_get(t, okey(l, lv[4 * i + 1], lv[4 * i + 2], lv[4 * i + 3])) >= 0) { *out = t; return -4; }
        leaf_append(t, l, lv[4 * i + 1], lv[4 * i + 2], lv[4 * i + 3]);
        vol += ldexpl(1.0L, -3 * (int)l);
    }
    *out = t;
    if (vol != 1.0L) return -4;
    for (int64_t i = 0; i < n; i++) {                     /* no leaf strictly inside another */
        orc_leaf o = t->leaves[i];
        for (int ll = (int)o.level - 1; ll >= 0; ll--) {
            int sh = (int)o.level - ll;
            if (hash_get(t, okey(ll, o.ix >> sh, o.iy >> sh, o.iz >> sh)) >= 0) return -4;
        }
    }
    int64_t before = t->used;
    balance(t);
    if (t->used != before) return -3;
    tree_finalise(t);
    return t->n;
}

int64_t orc_tree_size(const void *tv) { return ((const orc_tree *)tv)->n; }

void orc_tree_leaves(const void *tv, uint32_t *out)
{
    const orc_tree *t = (const orc_tree *)tv;
    memcpy(out, t->leaves, (size_t)t->n * sizeof(orc_leaf));
}

void orc_tree_free(void *tv)
{
    orc_tree *t = (orc_tree *)tv;
    if (!t) return;
    free(t->leaves); free(t->alive); free(t->hkey); free(t->hval); free(t);
}

/* ------------------------------------------------------------------ point location */

/* leaf containing lattice point P (per-axis index on the level-lq lattice, already wrapped) */
static int64_t locate(const orc_tree *t, int lq, const int64_t P[3])
{
    int64_t found = -1;
    for (int ll = 0; ll <= MAXLEVEL; ll++) {
        uint32_t c[3];
        for (int d = 0; d < 3; d++)
            c[d] = (uint32_t)(ll <= lq ? (P[d] >> 3) >> (lq - ll) : (P[d] << (ll - lq)) >> 3);
        int64_t i = hash_get(t, okey((uint32_t)ll, c[0], c[1], c[2]));
        if (i >= 0) { found = i; break; }   /* leaves are disjoint: at most one level can hit */
    }
    return found;
}

/* ------------------------------------------------------------------ Lagrange interpolation */

/* 256 * weights of the six-point Lagrange interpolant on nodes 0..5 evaluated at r = 1/2, 3/2,
 * ..., 11/2 (the last one extrapolates half a cell beyond node 5). */
static const double LAG256[6][6] = {
    {  63.0,  315.0, -210.0,  126.0,   -45.0,   7.0 },
    {  -7.0,  105.0,  210.0,  -70.0,    21.0,  -3.0 },
    {   3.0,  -25.0,  150.0,  150.0,   -25.0,   3.0 },
    {  -3.0,   21.0,  -70.0,  210.0,   105.0,  -7.0 },
    {   7.0,  -45.0,  126.0, -210.0,   315.0,  63.0 },
    { -63.0,  385.0, -990.0, 1386.0, -1155.0, 693.0 },
};

/* for an odd fine coordinate f in [1,15]: first coarse node s of the stencil and the row index */
static void lag_row(int f, int *s, int *row)
{
    int c0 = (f - 1) / 2;               /* coarse node just below the point */
    int st = c0 - 2; if (st < 0) st = 0; if (st > 2) st = 2;
    *s = st; *row = c0 - st;            /* r = c0 + 1/2 - s  ->  row = r - 1/2 */
}

static double lag_chain(const double v[6], int row)
{
    double acc = (LAG256[row][0] / 256.0) * v[0];
    for (int m = 1; m < 6; m++) acc = fma(LAG256[row][m] / 256.0, v[m], acc);
    return acc;
}

/* value at fine coordinates (fx,fy,fz) in [0,16)^3 inside a coarse leaf whose 8^3 nodes are src */
static double interp_x(const double *src, int fx, int cy, int cz)
{
    if (!(fx & 1)) return src[(cz * NPT + cy) * NPT + fx / 2];
    int s, row; double v[6];
    lag_row(fx, &s, &row);
    for (int m = 0; m < 6; m++) v[m] = src[(cz * NPT + cy) * NPT + s + m];
    return lag_chain(v, row);
}
static double interp_xy(const double *src, int fx, int fy, int cz)
{
    if (!(fy & 1)) return interp_x(src, fx, fy / 2, cz);
    int s, row; double v[6];
    lag_row(fy, &s, &row);
    for (int m = 0; m < 6; m++) v[m] = interp_x(src, fx, s + m, cz);
    return lag_chain(v, row);
}
static double interp_xyz(const double *src, int fx, int fy, int fz)
{
    if (!(fz & 1)) return interp_xy(src, fx, fy, fz / 2);
    int s, row; double v[6];
    lag_row(fz, &s, &row);
    for (int m = 0; m < 6; m++) v[m] = interp_xy(src, fx, fy, s + m);
    return lag_chain(v, row);
}

/* ------------------------------------------------------------------ unzip */

static int64_t sel_block(const int64_t *blocks, int64_t s) { return blocks ? blocks[s] : s; }

/* zipped [nvar][n][8][8][8] (all blocks)  ->  padded [nvar][nsel][14][14][14] (selected blocks,
 * in selection order; blocks==NULL means all blocks, nsel==n). */
void orc_unzip(const void *tv, int nvar, const double *zipped, double *padded, const int64_t *blocks, int64_t nsel)
{
    const orc_tree *t = (const orc_tree *)tv;
#pragma omp parallel for schedule(dynamic)
    for (int64_t s = 0; s < nsel; s++) {
        int64_t b = sel_block(blocks, s);
        orc_leaf B = t->leaves[b];
        int l = (int)B.level; int64_t N = (int64_t)NPT << l;
        const int64_t a[3] = { B.ix, B.iy, B.iz };
        for (int kk = 0; kk < NP; kk++) for (int jj = 0; jj < NP; jj++) for (int ii = 0; ii < NP; ii++) {
            const int pp[3] = { ii, jj, kk };
            int64_t P[3];
            for (int d = 0; d < 3; d++) P[d] = ((NPT * a[d] + pp[d] - PAD) % N + N) % N;
            int64_t L = locate(t, l, P);
            orc_leaf S = t->leaves[L];
            const int64_t sa[3] = { S.ix, S.iy, S.iz };
            int dl = (int)S.level - l;
            size_t po = ((size_t)kk * NP + jj) * NP + ii;
            for (int v = 0; v < nvar; v++) {
                const double *src = zipped + ((size_t)v * t->n + L) * BLK;
                double val;
                if (dl == 0) {
                    int q[3]; for (int d = 0; d < 3; d++) q[d] = (int)(P[d] - NPT * sa[d]);
                    val = src[(q[2] * NPT + q[1]) * NPT + q[0]];
                } else if (dl == 1) {
                    int q[3]; for (int d = 0; d < 3; d++) q[d] = (int)(2 * P[d] - NPT * sa[d]);
                    val = src[(q[2] * NPT + q[1]) * NPT + q[0]];
                } else if (dl == -1) {
                    int f[3]; for (int d = 0; d < 3; d++) f[d] = (int)(P[d] - 2 * NPT * sa[d]);
                    val = interp_xyz(src, f[0], f[1], f[2]);
                } else {
                    val = NAN;  /* cannot happen on a 26-balanced tree */
                }
                padded[((size_t)v * nsel + s) * PBLK + po] = val;
            }
        }
    }
}

/* ------------------------------------------------------------------ unzip, centred variant */

/* Variant of the ghost rule for a point whose containing leaf L is one level coarser: instead of
 * the clamped stencil on L's own 8 nodes, every odd fine coordinate f uses the CENTRED six-point
 * stencil on the coarse lattice, nodes c0-2 .. c0+3 with c0 = (f-1)/2, weights
 * (3, -25, 150, 150, -25, 3)/256.  Nodes outside L's own range 0..7 are ghost points of L, so the
 * values come from L's PADDED block (local index c+3), which must have been filled before: blocks
 * are processed coarsest level first.  Even coordinates pass through; x, then y, then z; the same
 * acc = w0*v0, acc = fma(w_m, v_m, acc) chain.  Copies and injections are as in orc_unzip. */
static double cen_chain(const double v[6])
{
    double acc = (LAG256[2][0] / 256.0) * v[0];
    for (int m = 1; m < 6; m++) acc = fma(LAG256[2][m] / 256.0, v[m], acc);
    return acc;
}
/* pad = L's padded block (14^3); c* are L-local coarse indices in [-3, 10] */
static double cen_x(const double *pad, int fx, int cy, int cz)
{
    const double *row = pad + ((size_t)(cz + PAD) * NP + (cy + PAD)) * NP + PAD;
    if (!(fx & 1)) return row[fx / 2];
    int c0 = (fx - 1) / 2; double v[6];
    for (int m = 0; m < 6; m++) v[m] = row[c0 - 2 + m];
    return cen_chain(v);
}
static double cen_xy(const double *pad, int fx, int fy, int cz)
{
    if (!(fy & 1)) return cen_x(pad, fx, fy / 2, cz);
    int c0 = (fy - 1) / 2; double v[6];
    for (int m = 0; m < 6; m++) v[m] = cen_x(pad, fx, c0 - 2 + m, cz);
    return cen_chain(v);
}
static double cen_xyz(const double *pad, int fx, int fy, int fz)
{
    if (!(fz & 1)) return cen_xy(pad, fx, fy, fz / 2);
    int c0 = (fz - 1) / 2; double v[6];
    for (int m = 0; m < 6; m++) v[m] = cen_xy(pad, fx, fy, c0 - 2 + m);
    return cen_chain(v);
}

/* zipped [nvar][n][8^3] -> padded [nvar][n][14^3], all blocks (a block needs the padded blocks of
 * coarser leaves, so there is no selection). */
void orc_unzip_centred(const void *tv, int nvar, const double *zipped, double *padded)
{
    const orc_tree *t = (const orc_tree *)tv;
    for (int lev = 0; lev <= MAXLEVEL; lev++) {
#pragma omp parallel for schedule(dynamic)
        for (int64_t b = 0; b < t->n; b++) {
            orc_leaf B = t->leaves[b];
            if ((int)B.level != lev) continue;
            int64_t N = (int64_t)NPT << lev;
            const int64_t a[3] = { B.ix, B.iy, B.iz };
            for (int kk = 0; kk < NP; kk++) for (int jj = 0; jj < NP; jj++) for (int ii = 0; ii < NP; ii++) {
                const int pp[3] = { ii, jj, kk };
                int64_t P[3];
                for (int d = 0; d < 3; d++) P[d] = ((NPT * a[d] + pp[d] - PAD) % N + N) % N;
                int64_t L = locate(t, lev, P);
                orc_leaf S = t->leaves[L];
                const int64_t sa[3] = { S.ix, S.iy, S.iz };
                int dl = (int)S.level - lev;
                size_t po = ((size_t)kk * NP + jj) * NP + ii;
                for (int v = 0; v < nvar; v++) {
                    const double *src = zipped + ((size_t)v * t->n + L) * BLK;
                    double val;
                    if (dl == 0) {
                        int q[3]; for (int d = 0; d < 3; d++) q[d] = (int)(P[d] - NPT * sa[d]);
                        val = src[(q[2] * NPT + q[1]) * NPT + q[0]];
                    } else if (dl == 1) {
                        int q[3]; for (int d = 0; d < 3; d++) q[d] = (int)(2 * P[d] - NPT * sa[d]);
                        val = src[(q[2] * NPT + q[1]) * NPT + q[0]];
                    } else if (dl == -1) {
                        int f[3]; for (int d = 0; d < 3; d++) f[d] = (int)(P[d] - 2 * NPT * sa[d]);
                        val = cen_xyz(padded + ((size_t)v * t->n + L) * PBLK, f[0], f[1], f[2]);
                    } else {
                        val = NAN;
                    }
                    padded[((size_t)v * t->n + b) * PBLK + po] = val;
                }
            }
        }
    }
}

/* padded [nvar][nsel][14^3] -> zipped [nvar][nsel][8^3]: strip the ghost layers */
void orc_zip(int nvar, int64_t nsel, const double *padded, double *zipped)
{
    for (int64_t q = 0; q < (int64_t)nvar * nsel; q++)
        for (int k = 0; k < NPT; k++) for (int j = 0; j < NPT; j++) for (int i = 0; i < NPT; i++)
            zipped[q * BLK + (k * NPT + j) * NPT + i] =
                padded[q * PBLK + ((size_t)(k + PAD) * NP + (j + PAD)) * NP + (i + PAD)];
}

/* Ghost-source table by point location: for block b and direction (dx,dy,dz) in {-1,0,1}^3
 * (index (dz+1)*9+(dy+1)*3+(dx+1)), entry = {kind, id0, id1, id2, id3}: the distinct leaves that
 * hold the points of that part of the padded block, ascending, -1 filled.  out is [n][27][5]. */
int orc_ghost_table(const void *tv, int32_t *out)
{
    const orc_tree *t = (const orc_tree *)tv;
    int bad = 0;
#pragma omp parallel for schedule(dynamic) reduction(+:bad)
    for (int64_t b = 0; b < t->n; b++) {
        orc_leaf B = t->leaves[b];
        int l = (int)B.level; int64_t N = (int64_t)NPT << l;
        const int64_t a[3] = { B.ix, B.iy, B.iz };
        for (int dir = 0; dir < 27; dir++) {
            int dlt[3] = { dir % 3 - 1, (dir / 3) % 3 - 1, dir / 9 - 1 };
            int lo[3], hi[3];
            for (int d = 0; d < 3; d++) {
                lo[d] = dlt[d] < 0 ? 0 : (dlt[d] == 0 ? PAD : PAD + NPT);
                hi[d] = dlt[d] < 0 ? PAD : (dlt[d] == 0 ? PAD + NPT : NP);
            }
            int64_t ids[8]; int nid = 0; int kind = -1;
            for (int kk = lo[2]; kk < hi[2]; kk++) for (int jj = lo[1]; jj < hi[1]; jj++) for (int ii = lo[0]; ii < hi[0]; ii++) {
                const int pp[3] = { ii, jj, kk };
                int64_t P[3];
                for (int d = 0; d < 3; d++) P[d] = ((NPT * a[d] + pp[d] - PAD) % N + N) % N;
                int64_t L = locate(t, l, P);
                int dl = (int)t->leaves[L].level - l;
                int k = dl == 0 ? G_SAME : (dl == 1 ? G_FINER : (dl == -1 ? G_COARSER : 99));
                if (kind < 0) kind = k;
                if (k != kind || k == 99) bad++;
                int seen = 0;
                for (int q = 0; q < nid; q++) if (ids[q] == L) seen = 1;
                if (!seen) { if (nid < 8) ids[nid++] = L; else bad++; }
            }
            for (int p = 1; p < nid; p++)                  /* insertion sort ascending */
                for (int q = p; q > 0 && ids[q] < ids[q - 1]; q--) { int64_t tmp = ids[q]; ids[q] = ids[q - 1]; ids[q - 1] = tmp; }
            if (nid > 4) bad++;
            int32_t *e = out + ((size_t)b * 27 + dir) * 5;
            e[0] = kind;
            for (int q = 0; q < 4; q++) e[1 + q] = q < nid ? (int32_t)ids[q] : -1;
        }
    }
    return bad;
}

/* ------------------------------------------------------------------ stencils */

#define C60  0x1.1111111111111p-6   /* 1/60  */
#define C180 0x1.6c16c16c16c17p-8   /* 1/180 */

/* first derivative from the six off-centre taps; ih = 1/h */
static double d1_taps(double m3, double m2, double m1, double p1, double p2, double p3, double ih)
{
    double d1 = p1 - m1, d2 = p2 - m2, d3 = p3 - m3;
    double t = fma(-9.0, d2, d3);
    t = fma(45.0, d1, t);
    return (t * C60) * ih;
}
/* second derivative; ih2 = 1/h^2 */
static double d2_taps(double m3, double m2, double m1, double u0, double p1, double p2, double p3, double ih2)
{
    double s1 = p1 + m1, s2 = p2 + m2, s3 = p3 + m3;
    double t = 2.0 * s3;
    t = fma(-27.0, s2, t);
    t = fma(270.0, s1, t);
    t = fma(-490.0, u0, t);
    return (t * C180) * ih2;
}
/* undivided sixth difference along one axis */
static double ko_taps(double m3, double m2, double m1, double u0, double p1, double p2, double p3)
{
    double s1 = p1 + m1, s2 = p2 + m2, s3 = p3 + m3;
    double q = fma(-6.0, s2, s3);
    q = fma(15.0, s1, q);
    q = fma(-20.0, u0, q);
    return q;
}

static const int STRIDE[3] = { 1, NP, NP * NP };

static double D1(const double *U, int c, int axis, double ih)
{
    int s = STRIDE[axis];
    return d1_taps(U[c - 3 * s], U[c - 2 * s], U[c - s], U[c + s], U[c + 2 * s], U[c + 3 * s], ih);
}
static double D2(const double *U, int c, int axis, double ih2)
{
    int s = STRIDE[axis];
    return d2_taps(U[c - 3 * s], U[c - 2 * s], U[c - s], U[c], U[c + s], U[c + 2 * s], U[c + 3 * s], ih2);
}
/* mixed derivative D1_a( D1_b U ), a = outer axis, b = inner axis */
static double DMIX(const double *U, int c, int a, int b, double ih)
{
    int s = STRIDE[a];
    return d1_taps(D1(U, c - 3 * s, b, ih), D1(U, c - 2 * s, b, ih), D1(U, c - s, b, ih),
                   D1(U, c + s, b, ih), D1(U, c + 2 * s, b, ih), D1(U, c + 3 * s, b, ih), ih);
}
static double KO(const double *U, int c, double sigma, double ih)
{
    double q[3];
    for (int a = 0; a < 3; a++) {
        int s = STRIDE[a];
        q[a] = ko_taps(U[c - 3 * s], U[c - 2 * s], U[c - s], U[c], U[c + s], U[c + 2 * s], U[c + 3 * s]);
    }
    return sigma * (((q[0] + q[1]) + q[2]) * (ih * 0.015625));
}
static double LAP(const double *U, int c, double ih2)
{
    return (D2(U, c, 0, ih2) + D2(U, c, 1, ih2)) + D2(U, c, 2, ih2);
}

int orc_nvar_in(int kind)  { return kind == ORC_DERIVS ? 1 : kind == ORC_WAVE ? 2 : kind == ORC_BURGERS ? 1 : kind == ORC_SYN24 ? 24 : -1; }
int orc_nvar_out(int kind) { return kind == ORC_DERIVS ? 4 : kind == ORC_WAVE ? 2 : kind == ORC_BURGERS ? 1 : kind == ORC_SYN24 ? 24 : -1; }

/* ------------------------------------------------------------------ right-hand sides */

/* One padded block: in[v] -> out[w] (padded-shaped, interior written only).
 * DERIVS : out = (D_x u, D_y u, D_z u, Laplacian u)
 * WAVE   : d_t u = pi + KO(u),  d_t pi = Laplacian u + KO(pi)
 * BURGERS: d_t u = -(u D_x u) + KO(u)                (paper, Eq. Inviscid_Burgers, 1-D flux along x)
 * SYN24  : 24 coupled fields, see syn24_point()      */
static void syn24_point(const double *const *in, double *const *out, int c, double sigma, double ih, double ih2)
{
    /* fields: 0 = alpha, 1..3 = beta^d, 4..9 = g_xx g_xy g_xz g_yy g_yz g_zz, 10..23 = others */
    double d[24][3], lap[10], ko[24];
    for (int a = 0; a < 24; a++) {
        for (int ax = 0; ax < 3; ax++) d[a][ax] = D1(in[a], c, ax, ih);
        ko[a] = KO(in[a], c, sigma, ih);
    }
    const double eps = 0.125;
    double Gxx = 1.0 - eps * in[4][c], Gxy = -(eps * in[5][c]), Gxz = -(eps * in[6][c]);
    double Gyy = 1.0 - eps * in[7][c], Gyz = -(eps * in[8][c]), Gzz = 1.0 - eps * in[9][c];
    for (int s = 0; s < 10; s++) {
        const double *U = in[s];
        double dxx = D2(U, c, 0, ih2), dyy = D2(U, c, 1, ih2), dzz = D2(U, c, 2, ih2);
        double dxy = DMIX(U, c, 0, 1, ih), dxz = DMIX(U, c, 0, 2, ih), dyz = DMIX(U, c, 1, 2, ih);
        double diag = Gxx * dxx; diag = fma(Gyy, dyy, diag); diag = fma(Gzz, dzz, diag);
        double off = Gxy * dxy; off = fma(Gxz, dxz, off); off = fma(Gyz, dyz, off);
        lap[s] = fma(2.0, off, diag);
    }
    double alpha = in[0][c], bx = in[1][c], by = in[2][c], bz = in[3][c];
    for (int a = 0; a < 24; a++) {
        int n = (a + 1) % 24, m = (a + 11) % 24;
        double kappa = ldexp(1.0, -(a % 4));
        double t1 = bx * d[a][0]; t1 = fma(by, d[a][1], t1); t1 = fma(bz, d[a][2], t1);
        double t2 = kappa * lap[a % 10];
        double t3 = d[a][0] * d[n][0]; t3 = fma(d[a][1], d[n][1], t3); t3 = fma(d[a][2], d[n][2], t3);
        t3 = 0.25 * t3;
        double t4 = (0.5 * alpha) * in[m][c];
        out[a][c] = (((t1 + t2) + t3) - t4) + ko[a];
    }
}

/* padded in [nvin][nsel][14^3] -> padded-shaped out [nvout][nsel][14^3], interior points only.
 * levels[s] = refinement level of selected block s (sets h). */
void orc_rhs(int kind, double sigma, int64_t nsel, const uint32_t *levels, const double *in, double *out)
{
    int nvi = orc_nvar_in(kind), nvo = orc_nvar_out(kind);
#pragma omp parallel for schedule(dynamic)
    for (int64_t s = 0; s < nsel; s++) {
        double ih = (double)((int64_t)NPT << levels[s]); /* 1/h = 2^(l+3), exact */
        double ih2 = ih * ih;
        const double *I[24]; double *O[24];
        for (int v = 0; v < nvi; v++) I[v] = in + ((size_t)v * nsel + s) * PBLK;
        for (int w = 0; w < nvo; w++) O[w] = out + ((size_t)w * nsel + s) * PBLK;
        for (int k = PAD; k < PAD + NPT; k++) for (int j = PAD; j < PAD + NPT; j++) for (int i = PAD; i < PAD + NPT; i++) {
            int c = (k * NP + j) * NP + i;
            switch (kind) {
            case ORC_DERIVS:
                O[0][c] = D1(I[0], c, 0, ih); O[1][c] = D1(I[0], c, 1, ih); O[2][c] = D1(I[0], c, 2, ih);
                O[3][c] = LAP(I[0], c, ih2);
                break;
            case ORC_WAVE:
                O[0][c] = I[1][c] + KO(I[0], c, sigma, ih);
                O[1][c] = LAP(I[0], c, ih2) + KO(I[1], c, sigma, ih);
                break;
            case ORC_BURGERS: {
                double flux = I[0][c] * D1(I[0], c, 0, ih);
                O[0][c] = KO(I[0], c, sigma, ih) - flux;
                break; }
            case ORC_SYN24:
                syn24_point(I, O, c, sigma, ih, ih2);
                break;
            }
        }
    }
}

/* F = zip(rhs(unzip(u))) for selected blocks: zipped_all [nvin][n][512] -> out [nvout][nsel][512].
 * Literal composition, done in chunks of blocks only to bound the padded temporaries. */
void orc_F(const void *tv, int kind, double sigma, const double *zipped_all, const int64_t *blocks, int64_t nsel, double *out)
{
    const orc_tree *t = (const orc_tree *)tv;
    int nvi = orc_nvar_in(kind), nvo = orc_nvar_out(kind);
    const int64_t CH = 256;
    double *pin = (double *)malloc((size_t)nvi * CH * PBLK * sizeof(double));
    double *pout = (double *)malloc((size_t)nvo * CH * PBLK * sizeof(double));
    double *zout = (double *)malloc((size_t)nvo * CH * BLK * sizeof(double));
    int64_t *ids = (int64_t *)malloc(CH * sizeof(int64_t));
    uint32_t *lev = (uint32_t *)malloc(CH * sizeof(uint32_t));
    for (int64_t s0 = 0; s0 < nsel; s0 += CH) {
        int64_t m = nsel - s0 < CH ? nsel - s0 : CH;
        for (int64_t q = 0; q < m; q++) { ids[q] = sel_block(blocks, s0 + q); lev[q] = t->leaves[ids[q]].level; }
        orc_unzip(t, nvi, zipped_all, pin, ids, m);
        memset(pout, 0, (size_t)nvo * m * PBLK * sizeof(double));
        orc_rhs(kind, sigma, m, lev, pin, pout);
        orc_zip(nvo, m, pout, zout);
        for (int w = 0; w < nvo; w++)
            memcpy(out + ((size_t)w * nsel + s0) * BLK, zout + (size_t)w * m * BLK, (size_t)m * BLK * sizeof(double));
    }
    free(pin); free(pout); free(zout); free(ids); free(lev);
}

/* Classical RK4 on the whole zipped state u [nvar][n][512], in place (kinds with nvin == nvout).
 *   k1 = F(u), k2 = F(u + dt/2 k1), k3 = F(u + dt/2 k2), k4 = F(u + dt k3),
 *   u <- u + dt/6 (((k1 + 2 k2) + 2 k3) + k4);  each a*k + u is one fma. */
int orc_rk4_step(const void *tv, int kind, double sigma, double dt, double *u)
{
    const orc_tree *t = (const orc_tree *)tv;
    int nv = orc_nvar_in(kind);
    if (nv != orc_nvar_out(kind)) return -1;
    size_t len = (size_t)nv * t->n * BLK;
    double *k = (double *)malloc(len * sizeof(double));
    double *acc = (double *)malloc(len * sizeof(double));
    double *st = (double *)malloc(len * sizeof(double));
    const double half = 0.5 * dt, sixth = dt / 6.0;
    orc_F(t, kind, sigma, u, NULL, t->n, k);                         /* k1 */
    for (size_t i = 0; i < len; i++) { acc[i] = k[i]; st[i] = fma(half, k[i], u[i]); }
    orc_F(t, kind, sigma, st, NULL, t->n, k);                        /* k2 */
    for (size_t i = 0; i < len; i++) { acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(half, k[i], u[i]); }
    orc_F(t, kind, sigma, st, NULL, t->n, k);                        /* k3 */
    for (size_t i = 0; i < len; i++) { acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(dt, k[i], u[i]); }
    orc_F(t, kind, sigma, st, NULL, t->n, k);                        /* k4 */
    for (size_t i = 0; i < len; i++) u[i] = fma(sixth, acc[i] + k[i], u[i]);
    free(k); free(acc); free(st);
    return 0;
}

/* The same two with the centred ghost rule: F = zip(rhs(unzip_centred(u))) on all blocks. */
void orc_F_centred(const void *tv, int kind, double sigma, const double *zipped_all, double *out)
{
    const orc_tree *t = (const orc_tree *)tv;
    int nvi = orc_nvar_in(kind), nvo = orc_nvar_out(kind);
    double *pin = (double *)malloc((size_t)nvi * t->n * PBLK * sizeof(double));
    double *pout = (double *)calloc((size_t)nvo * t->n * PBLK, sizeof(double));
    uint32_t *lev = (uint32_t *)malloc(t->n * sizeof(uint32_t));
    for (int64_t b = 0; b < t->n; b++) lev[b] = t->leaves[b].level;
    orc_unzip_centred(t, nvi, zipped_all, pin);
    orc_rhs(kind, sigma, t->n, lev, pin, pout);
    orc_zip(nvo, t->n, pout, out);
    free(pin); free(pout); free(lev);
}

int orc_rk4_step_centred(const void *tv, int kind, double sigma, double dt, double *u)
{
    const orc_tree *t = (const orc_tree *)tv;
    int nv = orc_nvar_in(kind);
    if (nv != orc_nvar_out(kind)) return -1;
    size_t len = (size_t)nv * t->n * BLK;
    double *k = (double *)malloc(len * sizeof(double));
    double *acc = (double *)malloc(len * sizeof(double));
    double *st = (double *)malloc(len * sizeof(double));
    const double half = 0.5 * dt, sixth = dt / 6.0;
    orc_F_centred(t, kind, sigma, u, k);                             /* k1 */
    for (size_t i = 0; i < len; i++) { acc[i] = k[i]; st[i] = fma(half, k[i], u[i]); }
    orc_F_centred(t, kind, sigma, st, k);                            /* k2 */
    for (size_t i = 0; i < len; i++) { acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(half, k[i], u[i]); }
    orc_F_centred(t, kind, sigma, st, k);                            /* k3 */
    for (size_t i = 0; i < len; i++) { acc[i] = acc[i] + 2.0 * k[i]; st[i] = fma(dt, k[i], u[i]); }
    orc_F_centred(t, kind, sigma, st, k);                            /* k4 */
    for (size_t i = 0; i < len; i++) u[i] = fma(sixth, acc[i] + k[i], u[i]);
    free(k); free(acc); free(st);
    return 0;
}

/* ------------------------------------------------------------------ inter-grid transfer */

/* Carry zipped data from one tree to another (the step after a regrid).  Every owned point of
 * every leaf of the target tree, lattice point P of that leaf's level l, takes the value the
 * source discretisation has at that place; with (l', a') the source leaf that contains it:
 *   l' >= l   the point is node 2^(l'-l) P - 8a' of that leaf: copy it (injection when l' > l);
 *   l' = l-1  interpolate inside that leaf exactly as for a ghost point taken from a coarser
 *             leaf: fine coordinate f = P - 16a' per axis, even f passes through, odd f uses the
 *             clamped six-point Lagrange row; x, then y, then z;
 *   l' < l-1  not defined here: the function returns -8 and writes nothing.
 * zipped_src [nvar][n_src][8^3] -> zipped_dst [nvar][n_dst][8^3]. */
int orc_transfer(const void *srcv, const void *dstv, int nvar, const double *zipped_src, double *zipped_dst)
{
    const orc_tree *S = (const orc_tree *)srcv, *D = (const orc_tree *)dstv;
    for (int64_t b = 0; b < D->n; b++) {       /* a target leaf lies inside one source leaf or covers whole ones */
        orc_leaf B = D->leaves[b];
        const int64_t P[3] = { NPT * (int64_t)B.ix, NPT * (int64_t)B.iy, NPT * (int64_t)B.iz };
        int64_t L = locate(S, (int)B.level, P);
        if (L < 0 || (int)S->leaves[L].level < (int)B.level - 1) return -8;
    }
#pragma omp parallel for schedule(dynamic)
    for (int64_t b = 0; b < D->n; b++) {
        orc_leaf B = D->leaves[b];
        int l = (int)B.level;
        const int64_t a[3] = { B.ix, B.iy, B.iz };
        for (int k = 0; k < NPT; k++) for (int j = 0; j < NPT; j++) for (int i = 0; i < NPT; i++) {
            const int64_t P[3] = { NPT * a[0] + i, NPT * a[1] + j, NPT * a[2] + k };
            int64_t L = locate(S, l, P);
            orc_leaf Q = S->leaves[L];
            const int64_t sa[3] = { Q.ix, Q.iy, Q.iz };
            int dl = (int)Q.level - l;
            for (int v = 0; v < nvar; v++) {
                const double *src = zipped_src + ((size_t)v * S->n + L) * BLK;
                double val;
                if (dl >= 0) {
                    int q[3]; for (int d = 0; d < 3; d++) q[d] = (int)((P[d] << dl) - NPT * sa[d]);
                    val = src[(q[2] * NPT + q[1]) * NPT + q[0]];
                } else {
                    int f[3]; for (int d = 0; d < 3; d++) f[d] = (int)(P[d] - 2 * NPT * sa[d]);
                    val = interp_xyz(src, f[0], f[1], f[2]);
                }
                zipped_dst[((size_t)v * D->n + b) * BLK + (k * NPT + j) * NPT + i] = val;
            }
        }
    }
    return 0;
}

/* 1-D helpers exported for the closed-form tests: apply the operators to a 7-point line */
double orc_d1_line(const double *u7, double ih) { return d1_taps(u7[0], u7[1], u7[2], u7[4], u7[5], u7[6], ih); }
double orc_d2_line(const double *u7, double ih2) { return d2_taps(u7[0], u7[1], u7[2], u7[3], u7[4], u7[5], u7[6], ih2); }
double orc_ko_line(const double *u7) { return ko_taps(u7[0], u7[1], u7[2], u7[3], u7[4], u7[5], u7[6]); }
/* interpolate inside one coarse leaf: src 8^3, fine coords in [0,16) */
double orc_interp(const double *src, int fx, int fy, int fz) { return interp_xyz(src, fx, fy, fz); }
