/*
 * octfd.h -- C ABI of liboctfd: block finite-difference pipeline on a 2:1-balanced periodic
 * octree of 8^3-point fp64 blocks, for one AMD MI355X (gfx950).
 *
 * Where the definitions come from.  The paper this library accompanies states one governing
 * equation (inviscid Burgers, introduction, Eq. "Inviscid_Burgers" with the initial data of Eq.
 * "initial-condition") and says only that derivatives are taken with finite-difference kernels
 * (Sec. II-A, "Implementing the forward model") that must respect a CFL condition, suggesting
 * higher-order stencils in Sec. V.  It defines no octree, ghost exchange, stencil order,
 * dissipation or time integrator.  Each entry point below therefore states the textbook
 * definition it implements.
 *
 * Conventions
 *   - every function returns an int status: OT_OK (0) or a negative OT_E_* code; nothing throws,
 *     aborts or prints.  ot_strerror() names a code, ot_last_hip_error() gives the last hipError_t.
 *   - "host" pointers are ordinary memory; "device" pointers are HIP device memory on the current
 *     device.  The caller owns every data array and the workspace.  The library owns only ot_tree
 *     and the device copies of its index tables (released by octree_free).
 *   - device entry points only enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     default stream).  They do not synchronise and do not allocate, with two exceptions.  (1) The
 *     device copies of a tree's index tables are a cache inside the opaque handle, which the first
 *     device call on the tree fills (one hipMalloc and synchronous copies; this fails inside a
 *     stream capture).  Call octree_upload beforehand where that matters.  The device that was
 *     current then must be the current one in every later call on the tree (else
 *     OT_E_UNSUPPORTED).  (2) rhs_eval_zipped, which has no workspace argument, keeps the virtual
 *     blocks of its input (see there) in an array that belongs to the tree; its first call on a
 *     tree with level jumps allocates that array (a later call with more variables enlarges it).
 *     rk_step, rk_step_centred and rk_step_static never allocate once the tables are uploaded.
 *   - data arrays hold doubles and must be 8-byte aligned, workspaces 256-byte aligned
 *     (OT_E_BADARG otherwise).
 *   - calls that use the same tree, plan or workspace must not overlap in time.
 *   - layouts (x fastest): zipped  [var][block][k][j][i]     8*8*8   doubles per block and variable
 *                          padded  [var][block][kk][jj][ii]  14*14*14, (ii,jj,kk) = (i,j,k)+3
 *     blocks are stored in Morton order of their anchors (x least significant bit).
 *   - input and output arrays must not overlap, except u in rk_step.
 *   - device calls accept trees of fewer than 2^20 blocks (OT_E_UNSUPPORTED otherwise); the host
 *     calls have no such limit.
 */
#ifndef OCTFD_H
#define OCTFD_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    OT_OK = 0,
    OT_E_BADARG = -1,      /* null pointer, size or enum out of range                    */
    OT_E_NOMEM = -2,       /* host or device allocation failed                           */
    OT_E_UNBALANCED = -3,  /* leaf list violates the 26-neighbour 2:1 balance            */
    OT_E_INCOMPLETE = -4,  /* leaf list has a gap, an overlap or a duplicate             */
    OT_E_WORKSPACE = -5,   /* workspace smaller than rk_workspace_bytes()                */
    OT_E_HIP = -6,         /* a HIP call failed, see ot_last_hip_error()                 */
    OT_E_NODEVICE = -7,    /* no usable GPU                                              */
    OT_E_UNSUPPORTED = -8  /* e.g. rk_step on a kind whose input and output counts differ */
};

typedef struct ot_tree ot_tree;

/* Leaf (l, ix, iy, iz) covers [i*2^-l, (i+1)*2^-l) per axis of the periodic unit cube and owns the
 * 8^3 lattice points I = 8*i + {0..7} of the level-l lattice (N_l = 8*2^l points per axis, spacing
 * h_l = 2^-(l+3); point I of level l coincides with point 2I of level l+1). */
typedef struct { uint32_t level, ix, iy, iz; } ot_leaf;

typedef struct {
    uint32_t lmin, lmax;         /* 3 <= lmin <= lmax <= 19                                        */
    uint32_t npts;               /* number of seed points                                          */
    const uint32_t *pts_q20;     /* host, 3*npts coordinates on the 2^20 lattice                   */
    const uint32_t *radius_q20;  /* host, lmax-lmin radii R_l <= 2^21 for l = lmin .. lmax-1 (same lattice) */
    uint32_t points_per_dim;     /* must be 8                                                      */
    uint32_t pad;                /* must be 3                                                      */
    uint32_t periodic;           /* must be 1                                                      */
} ot_build_params;

typedef enum { OT_RHS_DERIVS = 0, OT_RHS_WAVE = 1, OT_RHS_BURGERS = 2, OT_RHS_SYN24 = 3 } ot_rhs_kind;

typedef struct { double ko_sigma; double reserved[7]; } ot_rhs_params;

/* Tree construction (host only; works without a GPU).
 * Start from all octants of level lmin; split an octant of level l < lmax when a seed point lies
 * closer than R_l to its closed box (squared distance in int64 on the 2^20 lattice, minimum over
 * the periodic images of the point, strict <); then split leaves until every leaf's 26 periodic
 * neighbours differ from it by at most one level (the minimal such refinement is unique); order
 * the leaves by Morton key; derive the ghost-source table.  *out receives a new tree. */
int octree_build(const ot_build_params *params, ot_tree **out);

/* Same tables from an explicit leaf list in any order.  Fails with OT_E_INCOMPLETE unless the
 * leaves tile the cube exactly once, with OT_E_UNBALANCED unless they are 26-balanced. */
int octree_from_leaves(const ot_leaf *leaves, size_t n, uint32_t pad, ot_tree **out);

int octree_num_blocks(const ot_tree *tree, int64_t *nb);

/* Copies the leaves, in storage (Morton) order, to host array out[cap]; cap >= number of blocks. */
int octree_get_leaves(const ot_tree *tree, ot_leaf *out, size_t cap);

/* Ghost-source table, host array out[cap] of int32, cap >= nb*27*5.  Entry [b][d][0..4] describes
 * the part of block b's padded box in direction d = (dz+1)*9 + (dy+1)*3 + (dx+1), d* in {-1,0,1}:
 * [0] = 0 same level, 1 finer, 2 coarser; [1..4] = source block ids in ascending order, -1 filled
 * (finer: 4 ids across a face, 2 along an edge, 1 at a corner).  Entry d = 13 is the block itself. */
int octree_get_ghost_table(const ot_tree *tree, int32_t *out, size_t cap);

/* Copies the index tables to the current device now (otherwise done by the first device call), and
 * resolves the address of the library's static scratch array on that device (see rk_step_static). */
int octree_upload(ot_tree *tree);

int octree_free(ot_tree *tree); /* NULL is allowed */

/* Number of variables a kind reads / writes: DERIVS 1/4, WAVE 2/2, BURGERS 1/1, SYN24 24/24. */
int ot_rhs_nvar_in(ot_rhs_kind kind);
int ot_rhs_nvar_out(ot_rhs_kind kind);

/* unzip: zipped_dev [nvar][nb][8^3] -> padded_dev [nvar][nb][14^3].
 * Each padded point is lattice point P = 8a + (ii,jj,kk) - 3 (mod N_l) of the block's level and
 * receives the value held by the leaf that contains it: a copy from a leaf of the same level, an
 * injection (fine index 2P - 8a') from a finer leaf, or, from a coarser leaf, per axis with
 * f = P - 16a' in [0,16): node f/2 if f is even, else 6-point Lagrange interpolation on that
 * leaf's own nodes s..s+5, s = clamp((f-1)/2 - 2, 0, 2).  Axes are interpolated in the order
 * x, y, z, each as acc = w0*v0, acc = fma(w_m, v_m, acc).
 * (Like rhs_eval_zipped, the call keeps the virtual blocks of its input in an array owned by the
 * tree, allocated by the first call that needs it; see there.) */
int unzip(const ot_tree *tree, int nvar, const double *zipped_dev, double *padded_dev, void *hip_stream);

/* rhs_eval: padded_dev [nvar_in][nb][14^3] -> rhs_padded_dev [nvar_out][nb][14^3]; only the 8^3
 * interior of each output block is written.  Sixth-order centred first and second derivatives,
 * mixed derivatives as D1_a(D1_b u), sixth-difference Kreiss-Oliger dissipation with strength
 * ko_sigma fused into the same pass.
 *   DERIVS : (D_x u, D_y u, D_z u, Laplacian u), no dissipation
 *   WAVE   : d_t u = pi + KO(u);  d_t pi = Laplacian u + KO(pi)
 *   BURGERS: d_t u = KO(u) - u D_x u            (the paper's equation, flux along x)
 *   SYN24  : 24-field synthetic system with 72 first and 60 second derivatives.  Fields 0 = alpha,
 *            1..3 = beta^d, 4..9 = g_xx g_xy g_xz g_yy g_yz g_zz; G_dd = 1 - g_dd/8, G_de = -g_de/8;
 *            for s < 10:  Lap_s = fma(2, off, diag),  diag = fma(Gzz,Dzz, fma(Gyy,Dyy, Gxx*Dxx)),
 *                         off = fma(Gyz,Dyz, fma(Gxz,Dxz, Gxy*Dxy))   of field s;
 *            RHS_a = (((t1 + t2) + t3) - t4) + KO(u_a)  with  n = (a+1) mod 24  and
 *              t1 = fma(beta_z, D_z u_a, fma(beta_y, D_y u_a, beta_x * D_x u_a)),
 *              t2 = 2^-(a mod 4) * Lap_{a mod 10},
 *              t3 = 0.25 * fma(D_z u_a, D_z u_n, fma(D_y u_a, D_y u_n, D_x u_a * D_x u_n)),
 *              t4 = (0.5 * alpha) * u_{(a+11) mod 24}.
 * Operator sequences (h = 2^-(l+3), d_k = u[+k]-u[-k], s_k = u[+k]+u[-k]):
 *   D1 = (fma(45,d1, fma(-9,d2, d3)) * (1/60)) / h;
 *   D2 = (fma(-490,u0, fma(270,s1, fma(-27,s2, 2*s3))) * (1/180)) / h^2;  Laplacian = (D2x+D2y)+D2z;
 *   KO = sigma * (((q_x+q_y)+q_z) / (64 h)),  q = fma(-20,u0, fma(15,s1, fma(-6,s2, s3))).
 * For SYN24 the call uses variables 10..19 of the output array as scratch while it runs (each is
 * overwritten with its final value before the call's work completes). */
int rhs_eval(const ot_tree *tree, ot_rhs_kind kind, const ot_rhs_params *params,
             const double *padded_dev, double *rhs_padded_dev, void *hip_stream);

/* zip: padded_dev [nvar][nb][14^3] -> zipped_dev [nvar][nb][8^3]; drops the ghost layers.
 * OT_E_UNSUPPORTED when nb * nvar exceeds 2^31 - 1 (one workgroup per block and variable). */
int zip(const ot_tree *tree, int nvar, const double *padded_dev, double *zipped_dev, void *hip_stream);

/* The three calls above fused: zipped in, zipped right-hand side out, no padded array in memory.
 * Bit-identical to zip(rhs_eval(unzip(.))).
 * How level jumps are handled: where the same-level neighbour octant of a block does not exist
 * because its parent L is a leaf, unzip's rule makes the ghost values there a function of L's data
 * and of the fine position inside L alone.  Such an octant ("virtual block") is therefore filled
 * once per call (those of its y rows and z planes that some block reads; the rest is never read
 * and not written), x then y then z exactly as unzip interpolates a ghost point, and
 * the blocks around it copy from it as from a neighbour of their own level.  The virtual blocks of
 * the input take nvar * (number of virtual blocks) * 4 KB in an array owned by the tree. */
int rhs_eval_zipped(const ot_tree *tree, ot_rhs_kind kind, const ot_rhs_params *params,
                    const double *zipped_dev, double *rhs_zipped_dev, void *hip_stream);

/* Classical fourth-order Runge-Kutta step of d_t u = F(u), F = zip(rhs_eval(unzip(.))):
 *   k1 = F(u), k2 = F(u + dt/2 k1), k3 = F(u + dt/2 k2), k4 = F(u + dt k3),
 *   u <- u + dt/6 (((k1 + 2 k2) + 2 k3) + k4),  every a*k + u evaluated as one fma.
 * u_zipped_dev [nvar][nb][8^3] is updated in place.  workspace_dev must hold at least
 * rk_workspace_bytes() bytes (three zipped state vectors and the virtual blocks of one, see
 * rhs_eval_zipped), be 256-byte aligned and not overlap u (OT_E_BADARG otherwise).
 * Ghost values at level jumps follow unzip's rule, whose outermost row extrapolates by half a
 * coarse cell.  That row makes level jumps unstable for wave propagation over many steps (the wave
 * system on a three-level tree, sigma = 0.4: max |u| grows past 1e9 by t = 1); for evolutions
 * use rk_step_centred below, which is stable there. */
int rk_workspace_bytes(const ot_tree *tree, ot_rhs_kind kind, size_t *bytes);
int rk_step(const ot_tree *tree, ot_rhs_kind kind, const ot_rhs_params *params, double dt,
            double *u_zipped_dev, void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): rk_step with its workspace in a static device array of
 * OT_STATIC_WORKSPACE_BYTES that the library's code object holds on every GPU it is loaded on,
 * until the process ends.  Same arithmetic and results as rk_step.  The call allocates nothing and
 * does not synchronise; octree_upload(tree) must have been called on the current device before
 * (OT_E_UNSUPPORTED otherwise), and rk_workspace_bytes(tree, kind) must not exceed
 * OT_STATIC_WORKSPACE_BYTES (OT_E_WORKSPACE otherwise; the wave system on a three-level tree of 800
 * blocks needs 25 MB, the 24-field system on the uniform 512-block tree 151 MB).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU race, even
 * on different trees or streams.  Nothing in the array needs clearing between calls (every word
 * a step reads it has written before). */
#define OT_STATIC_WORKSPACE_BYTES ((size_t)160 << 20)
int rk_step_static(const ot_tree *tree, ot_rhs_kind kind, const ot_rhs_params *params, double dt,
                   double *u_zipped_dev, void *hip_stream);

/* Variant of the ghost rule with centred interpolation stencils (level-ordered).  Identical to
 * unzip except for padded points whose containing leaf L is one level coarser: there every odd
 * fine coordinate f = P - 16a' uses the centred six-point stencil on the coarse lattice, nodes
 * c0-2 .. c0+3 with c0 = (f-1)/2 and weights (3, -25, 150, 150, -25, 3)/256, instead of the stencil
 * clamped to L's own eight nodes.  Nodes outside 0..7 are ghost points of L and are taken from L's
 * padded block (local index c+3), so blocks are filled coarsest level first (one launch per
 * level) and the result depends on more than one source leaf.  Same axis order and fma chain.
 * The interpolation error at a level jump is much smaller (no half-cell extrapolation) and level
 * jumps stay stable for wave propagation over long times.
 *
 * rk_step_centred is rk_step with F = zip(rhs_eval(unzip_centred(.))), bit-identical to that
 * composition.  It differs from rk_step only in how the virtual blocks (see rhs_eval_zipped) are
 * filled before each stage: with the centred stencils, level by level, each from the part of its
 * source leaf's padded block that it needs (gathered from the zipped vector and from the virtual
 * blocks of the level before).  Same stage kernels, same workspace (rk_centred_workspace_bytes
 * equals rk_workspace_bytes), and within a few per cent of rk_step's time. */
int unzip_centred(const ot_tree *tree, int nvar, const double *zipped_dev, double *padded_dev, void *hip_stream);
int rk_centred_workspace_bytes(const ot_tree *tree, ot_rhs_kind kind, size_t *bytes);
int rk_step_centred(const ot_tree *tree, ot_rhs_kind kind, const ot_rhs_params *params, double dt,
                    double *u_zipped_dev, void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* Regrid: the tree that follows the moved refinement centres is built with octree_build; a
 * transfer plan then carries zipped data from the old tree to the new one.  (The paper has no
 * adaptive mesh; this is the step that surrounds the time loop in any adaptive run.)
 *
 * regrid_plan (host only) relates every leaf of `to` to the leaves of `from`.  The plan keeps
 * copies of what it needs, so both trees may be freed while it lives.  Fails with
 * OT_E_UNSUPPORTED when some leaf of `to` is two or more levels finer than the leaf of `from` that
 * contains it (refine one level per regrid).
 *
 * regrid_table copies the plan to host array out[cap] of int32, cap >= 4 * (blocks of `to`):
 * per target leaf {kind, first source leaf, number of source leaves, child octant} with kind
 *   0  the same leaf exists in `from`: copy its block;
 *   1  the source leaf is one level coarser: the target leaf is its child octant
 *      (ox | oy<<1 | oz<<2) and every point is interpolated inside the source leaf exactly as a
 *      ghost point is in unzip (fine coordinate f = 8*o + i per axis; x, then y, then z);
 *   2  the target leaf is tiled by that many consecutive finer source leaves: point I of level l
 *      is node 2^(l'-l) I of the level-l' source leaf that contains it, and is copied (injection).
 *
 * regrid_transfer: from_zipped_dev [nvar][blocks of from][8^3] -> to_zipped_dev [nvar][blocks of
 * to][8^3] on the current device, asynchronously on hip_stream; the first call copies the plan's
 * tables to the device, synchronously.  The arrays must not overlap. */
typedef struct ot_transfer ot_transfer;
int regrid_plan(const ot_tree *from, const ot_tree *to, ot_transfer **out);
int regrid_table(const ot_transfer *plan, int32_t *out, size_t cap);
int regrid_transfer(ot_transfer *plan, int nvar, const double *from_zipped_dev, double *to_zipped_dev,
                    void *hip_stream);
int regrid_free(ot_transfer *plan); /* NULL is allowed */

const char *ot_strerror(int status);
int ot_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OCTFD_H */
