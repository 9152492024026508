/* Plain C11 client of the C ABI: includes the public header as C, links liboctfd.so, and exercises
 * the host-only entry points (no GPU needed).  Built and run by tests/test_library_host.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "octfd.h"

int main(void)
{
    /* one seed point at the centre of level-3 octant (4,4,4), radius half an octant edge: exactly
     * that octant splits (the predicate is strict), 512 - 1 + 8 leaves */
    const uint32_t s = 1u << 17, c = 4 * s + s / 2;
    const uint32_t pts[3] = { c, c, c };
    const uint32_t radius[1] = { s / 2 };
    ot_build_params p = { 3, 4, 1, pts, radius, 8, 3, 1 };
    ot_tree *tree = NULL;
    int rc = octree_build(&p, &tree);
    if (rc != OT_OK) { printf("octree_build: %s\n", ot_strerror(rc)); return 1; }
    int64_t nb = 0;
    if (octree_num_blocks(tree, &nb) != OT_OK) return 2;
    ot_leaf *leaves = (ot_leaf *)malloc((size_t)nb * sizeof(ot_leaf));
    int32_t *ghost = (int32_t *)malloc((size_t)nb * 27 * 5 * sizeof(int32_t));
    if (octree_get_leaves(tree, leaves, (size_t)nb) != OT_OK) return 3;
    if (octree_get_ghost_table(tree, ghost, (size_t)nb * 27 * 5) != OT_OK) return 4;
    if (octree_get_leaves(tree, leaves, (size_t)nb - 1) != OT_E_BADARG) return 5;   /* short buffer is refused */
    int64_t fine = 0;
    for (int64_t b = 0; b < nb; ++b) fine += leaves[b].level == 4;
    /* the same tree from its own leaf list, and a plan between the two (every leaf is copied) */
    ot_tree *again = NULL;
    if (octree_from_leaves(leaves, (size_t)nb, 3, &again) != OT_OK) return 6;
    ot_transfer *plan = NULL;
    if (regrid_plan(tree, again, &plan) != OT_OK) return 7;
    int32_t *table = (int32_t *)malloc((size_t)nb * 4 * sizeof(int32_t));
    if (regrid_table(plan, table, (size_t)nb * 4) != OT_OK) return 8;
    int64_t copies = 0;
    for (int64_t b = 0; b < nb; ++b) copies += table[4 * b] == 0 && table[4 * b + 1] == (int32_t)b;
    size_t ws = 0;
    if (rk_workspace_bytes(tree, OT_RHS_WAVE, &ws) != OT_OK) return 9;
    if (rk_workspace_bytes(tree, OT_RHS_DERIVS, &ws) != OT_E_UNSUPPORTED) return 10;   /* 1 in, 4 out: no RK step */
    if (ot_rhs_nvar_in(OT_RHS_SYN24) != 24 || ot_rhs_nvar_out(OT_RHS_DERIVS) != 4) return 11;
    printf("blocks %lld fine %lld copies %lld self %d\n", (long long)nb, (long long)fine, (long long)copies,
           (int)ghost[13 * 5 + 1]);
    free(table); free(ghost); free(leaves);
    if (regrid_free(plan) != OT_OK || octree_free(again) != OT_OK || octree_free(tree) != OT_OK) return 12;
    if (octree_free(NULL) != OT_OK) return 13;
    return 0;
}
