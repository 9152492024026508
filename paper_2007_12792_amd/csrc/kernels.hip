// gfx950 kernels of liboctfd.
//
// One workgroup of 512 threads (8 wavefronts) owns one block and one thread owns one of its 8^3
// points.  A ghost-padded 14^3 tile of ONE variable lives in LDS; variables are streamed through it.
// The tile is filled either from a padded array (plain copy) or straight from zipped storage
// through the ghost-source table (copy, injection, separable Lagrange interpolation staged in
// LDS): `unzip` writes that tile out, the fused right-hand-side kernels consume it in place and
// never materialise the padded array.  Where each of a thread's tile entries comes from is worked
// out once per block (the "fill plan") and reused for every variable.
//
// Mixed second derivatives D1_a(D1_b u) are not evaluated as 36-tap stencils: every thread
// publishes its own D1_y u and D1_z u in LDS, the 3-deep ghost positions are filled in
// cooperatively, and the outer operator then takes six taps from that array.
//
// Arithmetic follows one fixed IEEE sequence per formula (see octfd.h); the file is compiled with
// -ffp-contract=off, so a fused multiply-add happens exactly where fma() is written.
#include "fill.hpp"
#include "stencils.hpp"
#include "syn24.hpp"
#include "tile.hpp"

#include <type_traits>

namespace octfd {
namespace {

// ---------------------------------------------------------------- right-hand-side kernel

// LDS of the right-hand-side kernels (in doubles / words)
template <int KIND>
struct RhsLds {
    static constexpr int NBUF = KIND == OT_RHS_SYN24 ? 2 : 1;
    // the 24-field system keeps D1_z u and D1_y u of the variable in hand here (mixed derivatives)
    static constexpr int NW = KIND == OT_RHS_SYN24 ? WZ + WY : 1;
    // second derivatives (SYN24 only) read the edge slabs of the tile too
    static constexpr int NPLAN = KIND == OT_RHS_SYN24 ? PLAN_EDGE : PLAN_FACE;
    static constexpr int NPOINTS = KIND == OT_RHS_SYN24 ? NEDGE : NFACE;
    static constexpr bool PLAN_IN_REGS = KIND != OT_RHS_SYN24;
    static constexpr int NPLAN_SRC = PLAN_IN_REGS ? 1 : NPLAN * NTHREADS;
};

// The right-hand side (and Runge-Kutta stage update) of whole blocks, one block per workgroup, all its variables.
// Zipped input (ZIN): the tile is filled through the ghost table in which coarser neighbours appear as virtual
// blocks, which k_virtual or k_virtual_centred has filled before the launch, so every tile entry is a copy or an
// injection and no interpolation happens here; the two ghost rules differ only in which of the two kernels ran.
// (The 24-field system on zipped input runs k_rhs_pair instead.)
template <int KIND, bool ZIN, int EPI>
__global__ __launch_bounds__(NTHREADS, waves_per_simd(KIND)) void k_rhs(DeviceTree tr, RhsArgs a)
{
    using L = RhsLds<KIND>;
    __shared__ double tiles[L::NBUF * TILE];
    __shared__ double wyz[L::NW];
    __shared__ BlockInfo bi;
    __shared__ uint32_t plan_src[L::NPLAN_SRC];
    constexpr int NPLAN = L::NPLAN, NPOINTS = L::NPOINTS;
    constexpr bool PLAN_IN_REGS = L::PLAN_IN_REGS;

    const int64_t b = block_of_workgroup(blockIdx.x);
    if (b >= tr.nb) return;                          // uniform over the workgroup, like everything below

    const int tid = threadIdx.x;
    const int64_t nb = tr.nb;
    load_block_info(bi, tr, b, tid);
    __syncthreads();

    int i, j, k;
    point_of(tid, i, j, k);
    const int c = tidx(k + PAD, j + PAD, i + PAD);
    // byte offsets of this thread's point inside one variable's zipped array / inside a padded block
    const uint32_t o8 = ((uint32_t)b * BLK + (k * NPT + j) * NPT + i) * 8u;
    const uint32_t p8 = (((k + PAD) * NP + (j + PAD)) * NP + (i + PAD)) * 8u;
    // 1/h = 2^(l+3) and 1/h^2, built from the level as bit patterns in scalar registers (the level is the same
    // for the whole workgroup, which the compiler cannot see through the LDS copy)
    const int lvl = __builtin_amdgcn_readfirstlane((int)bi.level);
    const double ih = __longlong_as_double((long long)(1026 + lvl) << 52), ih2 = __longlong_as_double((long long)(1029 + 2 * lvl) << 52);
    const double sigma = a.sigma;

    FillPlan<NPLAN, PLAN_IN_REGS> fp;
    fp.src = plan_src;
    if (ZIN) make_plan_zipped<NPLAN, NPOINTS>(fp, bi, tid);
    else make_plan_padded<NPLAN, NPOINTS>(fp, tid);
    double pv[NPLAN];

    auto var_base = [&](int v) -> const double* {
        return ZIN ? a.in + (int64_t)v * nb * BLK : a.in + ((int64_t)v * nb + b) * PBLK;
    };
    auto virt_base = [&](int v) -> const double* {  // variable v's virtual blocks
        return ZIN ? a.virt + (int64_t)v * tr.n_virt * BLK : nullptr;
    };
    auto stage = [&](int v) {   // bring variable v into tile buffer 0 (barrier before and after)
        __syncthreads();
        prefetch<NPLAN, PLAN_FACE, ZIN>(pv, fp, var_base(v), tid, virt_base(v));
        store_tile<NPLAN, PLAN_FACE>(tiles, fp, pv, tid);
        __syncthreads();
    };
    auto centre = [&](int v) -> double {   // this thread's own value of variable v
        return ZIN ? ldg(a.in + (int64_t)v * nb * BLK, o8) : ldg(a.in + ((int64_t)v * nb + b) * PBLK, p8);
    };

    if (KIND == OT_RHS_DERIVS) {
        stage(0);
        const EpiOperands e0 = epi_prefetch<EPI>(a, nb, 0, o8), e1 = epi_prefetch<EPI>(a, nb, 1, o8);
        const EpiOperands e2 = epi_prefetch<EPI>(a, nb, 2, o8), e3 = epi_prefetch<EPI>(a, nb, 3, o8);
        const PointOps p = point_ops<true>(tiles, c, 0.0, ih, ih2);
        emit<EPI>(a, nb, 0, b, o8, p8, p.dx, e0);
        emit<EPI>(a, nb, 1, b, o8, p8, p.dy, e1);
        emit<EPI>(a, nb, 2, b, o8, p8, p.dz, e2);
        emit<EPI>(a, nb, 3, b, o8, p8, p.lap, e3);
    } else if (KIND == OT_RHS_WAVE) {
        stage(0);
        prefetch<NPLAN, PLAN_FACE, ZIN>(pv, fp, var_base(1), tid, virt_base(1));   // pi is on its way while u is differentiated
        const PointOps pu = point_ops<true>(tiles, c, sigma, ih, ih2);
        // the operands of the stage update are requested only now: four more values live during the stencils
        // above push the kernel over the 64 registers that let four workgroups share a compute unit, and a
        // kernel that spills there loses a quarter of its speed (the fence keeps the scheduler from moving the
        // loads back up)
        __syncthreads();
        store_tile<NPLAN, PLAN_FACE>(tiles, fp, pv, tid);
        __builtin_amdgcn_sched_barrier(0);
        const EpiOperands e0 = epi_prefetch<EPI, ZIN>(a, nb, 0, o8), e1 = epi_prefetch<EPI, ZIN>(a, nb, 1, o8);
        __syncthreads();
        const PointOps pp = point_ops<false>(tiles, c, sigma, ih, ih2);
        emit<EPI>(a, nb, 0, b, o8, p8, pp.u0 + pu.ko, ZIN ? with_u<EPI>(e0, pu.u0) : e0);
        emit<EPI>(a, nb, 1, b, o8, p8, pu.lap + pp.ko, ZIN ? with_u<EPI>(e1, pp.u0) : e1);
    } else if (KIND == OT_RHS_BURGERS) {
        stage(0);
        const EpiOperands e0 = epi_prefetch<EPI, ZIN>(a, nb, 0, o8);
        const PointOps p = point_ops<false>(tiles, c, sigma, ih, ih2);
        const double flux = p.u0 * p.dx;
        emit<EPI>(a, nb, 0, b, o8, p8, p.ko - flux, ZIN ? with_u<EPI>(e0, p.u0) : e0);
    } else {
        // SYN24.  The variables are streamed in descending cyclic order (see syn24_stream).  The
        // first ten real passes (variables 9..0) evaluate the second-derivative combinations Lap_s;
        // each thread parks them at its own point in variables 10+s of the `stash` array, from where
        // the later passes (variables 23..10, which need Lap_{a mod 10}) read them back before those
        // slots receive their final values.  Per-thread state thus shrinks to one gradient.
        //
        // The tile is double-buffered and global memory is requested ahead of its use: tile data
        // of the next variable is loaded into registers at the top of a pass and stored to the
        // other LDS buffer at its end (one barrier per pass, plus the one inside mixed_derivs); the
        // pointwise operands of the next pass (RK accumulator and state, u_{a+11}, Lap) likewise.
        double* wz = wyz;
        double* wy = wyz + WZ;
        const double halpha = 0.5 * centre(0), bx = centre(1), by = centre(2), bz = centre(3);
        const double Gxx = 1.0 - 0.125 * centre(4), Gxy = -(0.125 * centre(5)), Gxz = -(0.125 * centre(6));
        const double Gyy = 1.0 - 0.125 * centre(7), Gyz = -(0.125 * centre(8)), Gzz = 1.0 - 0.125 * centre(9);
        double nx = 0, ny = 0, nz = 0;
        const int ownz = k * PS + (j + PAD) * RS + (i + PAD), owny = k * YPS + j * RS + (i + PAD);
        struct Look { double unext, lap; EpiOperands eo; };

        auto stash_base = [&](int v) -> double* {   // where Lap_{v-10} is parked (v = 10..19)
            return EPI == kOutPadded ? a.stash + ((int64_t)v * nb + b) * PBLK : a.stash + (int64_t)v * nb * BLK;
        };
        const uint32_t s8 = EPI == kOutPadded ? p8 : o8;

        // top of pass t: request the tile data of pass t+1 and this pass's own pointwise operands.
        // NEXT_USE says how much of the tile pass t+1 reads (edges only if it takes second derivatives).
        auto issue = [&](int t, int f, Look& l, int& f1, auto next_use) {
            constexpr int NEXT_USE = decltype(next_use)::value;
            if (t + 1 < NSTREAM) {
                f1 = syn24_stream(t + 1);
                prefetch<NPLAN, NEXT_USE, ZIN>(pv, fp, var_base(f1), tid, virt_base(f1));
            }
            l.unext = centre((f + 11) % 24);
            l.eo = epi_prefetch<EPI>(a, nb, f, o8);
            if (t > 10) l.lap = ldg(stash_base(10 + f % 10), s8);
        };
        using UseEdge = std::integral_constant<int, PLAN_EDGE>;
        using UseFace = std::integral_constant<int, PLAN_FACE>;
        // pass over a variable with second derivatives (9..0)
        auto pass_d2 = [&](int t, auto next_use) {
            constexpr int NEXT_USE = decltype(next_use)::value;
            const double* T = tiles + (t & 1) * TILE;
            const int f = syn24_stream(t);
            int f1 = 0;
            Look l{0.0, 0.0, {0.0, 0.0}};
            issue(t, f, l, f1, next_use);
            const Syn24Part p = syn24_axes<true>(T, c, wy, wz, owny, ownz, nx, ny, nz, bx, by, bz, Gxx, Gyy, Gzz, sigma, ih, ih2);
            const Mixed mx = mixed_derivs(T, wy, wz, tid, owny, ownz, ih);
            double off = Gxy * mx.dxy;
            off = fma(Gxz, mx.dxz, off);
            off = fma(Gyz, mx.dyz, off);
            const double lap = fma(2.0, off, p.diag);
            stg(stash_base(10 + f), s8, lap);
            emit<EPI>(a, nb, f, b, o8, p8, syn24_combine(p, f, lap, halpha, l.unext), l.eo);
            store_tile<NPLAN, NEXT_USE>(tiles + ((t + 1) & 1) * TILE, fp, pv, tid);
            __syncthreads();
        };
        // pass over a variable without second derivatives (23..10)
        auto pass_light = [&](int t) {
            const double* T = tiles + (t & 1) * TILE;
            const int f = syn24_stream(t);
            int f1 = 0;
            Look l{0.0, 0.0, {0.0, 0.0}};
            issue(t, f, l, f1, UseFace{});
            const Syn24Part p = syn24_axes<false>(T, c, wy, wz, owny, ownz, nx, ny, nz, bx, by, bz, 0.0, 0.0, 0.0, sigma, ih, ih2);
            emit<EPI>(a, nb, f, b, o8, p8, syn24_combine(p, f, l.lap, halpha, l.unext), l.eo);
            if (t + 1 < NSTREAM) {
                store_tile<NPLAN, PLAN_FACE>(tiles + ((t + 1) & 1) * TILE, fp, pv, tid);
                __syncthreads();
            }
        };

        {   // pass 0: gradient of variable 10 only
            const int f = syn24_stream(0), f1 = syn24_stream(1);
            prefetch<NPLAN, PLAN_FACE, ZIN>(pv, fp, var_base(f), tid, virt_base(f));
            store_tile<NPLAN, PLAN_FACE>(tiles, fp, pv, tid);
            __syncthreads();
            prefetch<NPLAN, PLAN_EDGE, ZIN>(pv, fp, var_base(f1), tid, virt_base(f1));
            nx = d1_at(tiles, c, 1, ih); ny = d1_at(tiles, c, RS, ih); nz = d1_at(tiles, c, PS, ih);
            store_tile<NPLAN, PLAN_EDGE>(tiles + TILE, fp, pv, tid);
            __syncthreads();
        }
#pragma unroll 1
        for (int t = 1; t < 10; ++t) pass_d2(t, UseEdge{});
        pass_d2(10, UseFace{});
#pragma unroll 1
        for (int t = 11; t < NSTREAM; ++t) pass_light(t);
    }
}

// ---------------------------------------------------------------- unzip / zip kernels

// unzip as a gather.  With the virtual blocks of the input filled (by k_virtual for the clamped ghost rule, by
// k_virtual_centred for the centred one), every one of the 2,744 points of a padded block is a copy: of the block's
// own data, of a same-level or virtual neighbour, or of the coinciding node of a finer neighbour.  A thread owns up to
// six consecutive-by-512 output positions of the padded block and keeps their sources in registers for all
// variables; no LDS, no barrier, loads and stores of different variables overlap freely.  The stores are non-temporal:
// the padded output (5.4 times the input) is not read again here and would otherwise push the ghost rows out of the L2
// (23.8 -> 20.5 ms on the 102,075-block tree with 24 fields).
// Workgroup r + G b takes variables r, r + G, r + 2G, ... of block b, G = min(8, nvar): with the workgroups dealt to
// the eight XCDs in turn, an XCD sees a fixed subset of the variables for consecutive blocks one after the other, so a
// ghost row it fetches was, or soon will be, an interior row of a block it handles for the same variable and is
// served by its L2.
__global__ __launch_bounds__(NTHREADS) void k_unzip(DeviceTree tr, int nvar, const double* __restrict__ zipped, const double* __restrict__ virt,
                                                    double* __restrict__ padded)
{
    __shared__ int32_t gt[27 * 5];
    const int tid = threadIdx.x;
    const int stride = nvar < NXCD ? nvar : NXCD;
    const int64_t b = blockIdx.x / stride, nb = tr.nb;
    const int v0 = (int)(blockIdx.x - b * stride);
    if (tid < 27 * 5) gt[tid] = tr.ghost_v[b * (27 * 5) + tid];
    __syncthreads();
    uint32_t off[PLAN_FULL];
#pragma unroll
    for (int m = 0; m < PLAN_FULL; ++m) {
        const int p = min(tid + m * NTHREADS, PBLK - 1);
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        const int rx = ii < PAD ? 0 : (ii < PAD + NPT ? 1 : 2);
        const int ry = jj < PAD ? 0 : (jj < PAD + NPT ? 1 : 2);
        const int rz = kk < PAD ? 0 : (kk < PAD + NPT ? 1 : 2);
        const int lx = ii - PAD + (1 - rx) * NPT, ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
        off[m] = ghost_source(&gt[(rz * 9 + ry * 3 + rx) * 5], rx, ry, rz, lx, ly, lz);   // the centre entry is the block itself
    }
    // the loads of two variables are in flight before the first store (22.1 -> 20.3 ms; three gain nothing more)
    constexpr int FLIGHT = 2;
#pragma unroll 1
    for (int v = v0; v < nvar; v += FLIGHT * stride) {
        double pv[FLIGHT][PLAN_FULL];
#pragma unroll
        for (int g = 0; g < FLIGHT; ++g) {
            const int w = v + g * stride;
            if (w < nvar) {
                const double* base = zipped + (int64_t)w * nb * BLK;
                const double* vbase = virt + (int64_t)w * tr.n_virt * BLK;
#pragma unroll
                for (int m = 0; m < PLAN_FULL; ++m) pv[g][m] = ldg((off[m] & 1u) ? vbase : base, off[m] & ~1u);
            }
        }
#pragma unroll
        for (int g = 0; g < FLIGHT; ++g) {
            const int w = v + g * stride;
            if (w < nvar) {
                double* out = padded + ((int64_t)w * nb + b) * PBLK;
#pragma unroll
                for (int m = 0; m < PLAN_FULL; ++m) {
                    const int p = tid + m * NTHREADS;
                    if (p < PBLK) __builtin_nontemporal_store(pv[g][m], out + p);
                }
            }
        }
    }
}

// Virtual blocks.  A virtual block is a child octant o of its source leaf; its 8^3 points are the fine positions
// f = 8 o + i per axis inside the leaf, interpolated x, then y, then z like any ghost point that comes from a
// coarser leaf.  Here a LANE owns a whole line of a pass: it holds the line's eight coarse nodes in registers and
// produces its eight fine values (four pass through, four take the clamped six-point stencil; which ones is the
// same for all lanes, so the weights are constants).  A wavefront owns one variable of the block: its 64 lanes are
// the 64 lines of a pass, the passes hand over through a staging array of the wavefront's own, in place, and nothing
// needs a workgroup barrier.  The eight wavefronts of a workgroup take eight variables of one virtual block at a time
// (or, with fewer variables, of several virtual blocks).
// (The same passes with one thread per point were bound by LDS instructions: 1.3 ms per call on the 102,075-block tree.)

// the eight fine values r of a child half (O = 0 lower, 1 upper) of a line with nodes v: for odd f = 8 O + i the same
// sequence as interp_line (first node s = clamp(c0 - 2, 0, 2), c0 = (f - 1) / 2; acc = w0 v_s, then five fma)
template <int O>
__device__ __forceinline__ void fine_half_line(const double (&v)[8], double (&r)[8])
{
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        r[2 * n] = v[4 * O + n];
        constexpr int kLo = 0;
        const int c0 = 4 * O + n, s = c0 - 2 < kLo ? kLo : (c0 - 2 > 2 ? 2 : c0 - 2), row = c0 - s;
        double acc = c_lag[row * 6] * v[s];
#pragma unroll
        for (int m = 1; m < 6; ++m) acc = fma(c_lag[row * 6 + m], v[s + m], acc);
        r[2 * n + 1] = acc;
    }
}
__device__ __forceinline__ void fine_line(int o, const double (&v)[8], double (&r)[8])
{
    if (o) fine_half_line<1>(v, r);                  // uniform
    else fine_half_line<0>(v, r);
}

constexpr int VPS = 72;                              // plane stride of the staging array, 8 (mod 32): no bank conflicts in the y pass
__global__ __launch_bounds__(NTHREADS) void k_virtual(DeviceTree tr, int nvar, const double* __restrict__ zipped, double* __restrict__ virt)
{
    __shared__ double staging[8][NPT * VPS];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    // with fewer than eight variables a workgroup takes several virtual blocks, so that no wavefront idles:
    // wavefront w -> virtual block `sub` of the workgroup's `per`, variables v0, v0 + nv, ...
    const int nv = nvar < 8 ? nvar : 8, per = 8 / nv;
    const int sub = wave / nv, v0 = wave - sub * nv;
    // runs of 16 consecutive workgroups (the children of a few source leaves) go to one XCD, whose L2 then serves
    // the re-reads of a source leaf by its other children
    const int64_t q = block_of_workgroup(blockIdx.x) * per + sub, nb = tr.nb;
    if (sub >= per || q >= tr.n_virt) return;        // uniform over the wavefront; the kernel has no workgroup barrier
    const int64_t leaf = tr.vblk[2 * q];
    const int oct = tr.vblk[2 * q + 1];
    const int need = tr.vneed[q];                                // y rows and z planes that any block reads
    const int ox = oct & 1, oy = (oct >> 1) & 1, oz = oct >> 2;
    const int hi = lane >> 3, lo = lane & 7;
    const bool row_needed = (need >> hi) & 1;
    double* A = staging[wave];
    const int64_t in_stride = nb * BLK, out_stride = tr.n_virt * BLK;
    const double* in = zipped + leaf * BLK + lane * NPT;        // x pass: this lane's line is (cz, cy) = (hi, lo)
    double* out = virt + q * BLK + lane;                        // z pass: this lane's line is (ty, tx) = (hi, lo)
    double nxt[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) nxt[m] = in[v0 * in_stride + m];
#pragma unroll 1
    for (int v = v0; v < nvar; v += nv) {
        double c[8], r[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) c[m] = nxt[m];
        if (v + nv < nvar) {
#pragma unroll
            for (int m = 0; m < 8; ++m) nxt[m] = in[(v + nv) * in_stride + m];
        }
        fine_line(ox, c, r);                                    // (cz, cy) -> fine x
#pragma unroll
        for (int m = 0; m < 8; ++m) A[hi * VPS + lo * NPT + m] = r[m];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < 8; ++m) c[m] = A[hi * VPS + m * NPT + lo];      // line (cz, tx) = (hi, lo) over cy
        fine_line(oy, c, r);
        // in place: a lane writes exactly the positions it has just read
#pragma unroll
        for (int m = 0; m < 8; ++m) A[hi * VPS + m * NPT + lo] = r[m];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < 8; ++m) c[m] = A[m * VPS + lane];              // line (ty, tx) = (hi, lo) over cz
        fine_line(oz, c, r);
        // only the rows and planes that are read are written (whole x rows: 64-byte pieces)
#pragma unroll
        for (int m = 0; m < 8; ++m)
            if (row_needed && ((need >> (8 + m)) & 1)) out[v * out_stride + m * (NPT * NPT)] = r[m];
        __builtin_amdgcn_wave_barrier();                         // the next variable's x pass overwrites the array
    }
}

// Virtual blocks with the centred ghost rule.  The value at a fine position inside a leaf L that is one level coarser
// is the centred six-point stencil on the coarse lattice around it, nodes c0 - 2 .. c0 + 3 with c0 = f / 2, and nodes
// outside L are ghost points of L.  A child octant o of L therefore needs, per axis, the nine coarse nodes
// 4 o - 2 .. 4 o + 6: a 9^3 part of L's padded block, which is gathered here straight from the zipped array and from
// the virtual blocks of L's own level (a plan of 729 sources, made once per workgroup from L's table row and shared
// by all variables), so launches go level by level, coarsest first.  Then the same three passes as in k_virtual,
// with nine nodes per line (81, 72 and 64 lines: a lane takes a second line where there are more than 64).
constexpr int CN = 9;                                // coarse nodes per axis
constexpr int CRS = CN, CPS = CN * CN + 7;           // row and plane stride of a wavefront's staging array: 88 = 24 (mod 32)
constexpr int CSTAGE = CN * CPS;

// the eight fine values of a line with nine nodes v (node n is coarse node 4 o - 2 + n): even f passes node c0 through,
// odd f takes nodes c0 - 2 .. c0 + 3 with the centred weights, acc = w0 v, then five fma (as centred_line)
__device__ __forceinline__ void fine_line_centred(const double (&v)[CN], double (&r)[8])
{
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        r[2 * n] = v[n + 2];
        double acc = c_lag[12] * v[n];
#pragma unroll
        for (int m = 1; m < 6; ++m) acc = fma(c_lag[12 + m], v[n + m], acc);
        r[2 * n + 1] = acc;
    }
}

__global__ __launch_bounds__(NTHREADS) void k_virtual_centred(DeviceTree tr, const int32_t* __restrict__ list, int64_t nlist, int nvar,
                                                              const double* __restrict__ zipped, double* virt)
{
    __shared__ double staging[8][CSTAGE];
    __shared__ uint32_t plan[CN * CN * CN];          // byte offsets of the 729 sources, bit 0: virtual block
    __shared__ int32_t gt[27 * 5];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t w = block_of_workgroup(blockIdx.x), nb = tr.nb;
    if (w >= nlist) return;                          // uniform
    const int64_t q = list[w];
    const int64_t leaf = tr.vblk[2 * q];
    const int oct = tr.vblk[2 * q + 1];
    const int need = tr.vneed[q];                    // y rows and z planes that any block reads
    if (tid < 27 * 5) gt[tid] = tr.ghost_v[leaf * (27 * 5) + tid];
    __syncthreads();
    for (int p = tid; p < CN * CN * CN; p += NTHREADS) {
        const int nz = p / (CN * CN), r = p - nz * CN * CN, ny = r / CN, nx = r - ny * CN;
        // position in L's padded block: coarse node 4 o - 2 + n, shifted by the three ghost layers
        const int ii = 4 * (oct & 1) + 1 + nx, jj = 4 * ((oct >> 1) & 1) + 1 + ny, kk = 4 * (oct >> 2) + 1 + nz;
        const int rx = ii < PAD ? 0 : (ii < PAD + NPT ? 1 : 2);
        const int ry = jj < PAD ? 0 : (jj < PAD + NPT ? 1 : 2);
        const int rz = kk < PAD ? 0 : (kk < PAD + NPT ? 1 : 2);
        const int lx = ii - PAD + (1 - rx) * NPT, ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
        plan[p] = ghost_source(&gt[(rz * 9 + ry * 3 + rx) * 5], rx, ry, rz, lx, ly, lz);   // the centre entry is L itself
    }
    __syncthreads();
    double* A = staging[wave];
    const int hi = lane >> 3, lo = lane & 7;
    const int64_t in_stride = nb * BLK, out_stride = tr.n_virt * BLK;
    double* out = virt + q * BLK + lane;
    // this lane's share of the gather: elements lane, lane + 64, ... of the 729
    constexpr int NG = (CN * CN * CN + 63) / 64;     // 12
    uint32_t off[NG];
    int dst[NG];
#pragma unroll
    for (int m = 0; m < NG; ++m) {
        const int p = min(lane + 64 * m, CN * CN * CN - 1);
        const int nz = p / (CN * CN), r = p - nz * CN * CN, ny = r / CN;
        off[m] = plan[p];
        dst[m] = nz * CPS + ny * CRS + (r - ny * CN);
    }
    auto gather = [&](double (&g)[NG], int v) {
        const double* base = zipped + v * in_stride;
        const double* vbase = virt + v * out_stride;
#pragma unroll
        for (int m = 0; m < NG; ++m) g[m] = ldg((off[m] & 1u) ? vbase : base, off[m] & ~1u);
    };
    double nxt[NG];
    if (wave < nvar) gather(nxt, wave);
#pragma unroll 1
    for (int v = wave; v < nvar; v += 8) {
#pragma unroll
        for (int m = 0; m < NG; ++m) A[dst[m]] = nxt[m];         // the last element is stored twice by the lanes past 729
        if (v + 8 < nvar) gather(nxt, v + 8);
        __builtin_amdgcn_wave_barrier();
        double c[CN], r[8];
        // x pass: lines (cz, cy), 81 of them; in place (a lane writes the first eight positions of the row it has read)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int line = lane + 64 * h;
            if (line < CN * CN) {
                double* row = A + (line / CN) * CPS + (line % CN) * CRS;
#pragma unroll
                for (int m = 0; m < CN; ++m) c[m] = row[m];
                fine_line_centred(c, r);
#pragma unroll
                for (int m = 0; m < 8; ++m) row[m] = r[m];
            }
        }
        __builtin_amdgcn_wave_barrier();
        // y pass: lines (cz, tx), 72 of them; in place
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int line = lane + 64 * h;
            if (line < CN * 8) {
                double* col = A + (line >> 3) * CPS + (line & 7);
#pragma unroll
                for (int m = 0; m < CN; ++m) c[m] = col[m * CRS];
                fine_line_centred(c, r);
#pragma unroll
                for (int m = 0; m < 8; ++m) col[m * CRS] = r[m];
            }
        }
        __builtin_amdgcn_wave_barrier();
        // z pass: lines (ty, tx) = (hi, lo)
#pragma unroll
        for (int m = 0; m < CN; ++m) c[m] = A[m * CPS + hi * CRS + lo];
        fine_line_centred(c, r);
#pragma unroll
        for (int m = 0; m < 8; ++m)
            if (((need >> hi) & 1) && ((need >> (8 + m)) & 1)) out[v * out_stride + m * (NPT * NPT)] = r[m];
        __builtin_amdgcn_wave_barrier();                         // the next variable's gather overwrites the array
    }
}

__global__ __launch_bounds__(NTHREADS) void k_zip(int64_t nblocks, const double* __restrict__ padded, double* __restrict__ zipped)
{
    const int tid = threadIdx.x;
    const int64_t q = blockIdx.x;   // var*nb + block
    if (q >= nblocks) return;
    const int i = tid & 7, j = (tid >> 3) & 7, k = tid >> 6;
    zipped[q * BLK + tid] = padded[q * PBLK + ((k + PAD) * NP + (j + PAD)) * NP + (i + PAD)];
}

template <int KIND, bool ZIN, int EPI>
hipError_t launch_one(const DeviceTree& t, const RhsArgs& a, hipStream_t s)
{
    if constexpr (KIND == OT_RHS_SYN24 && ZIN) {
        return launch_rhs_pairs(t, static_cast<Epilogue>(EPI), a, s);
    } else {
        hipLaunchKernelGGL((k_rhs<KIND, ZIN, EPI>), dim3(grid_for_blocks(t.nb)), dim3(NTHREADS), 0, s, t, a);
        return hipGetLastError();
    }
}

template <int KIND>
hipError_t launch_kind(const DeviceTree& t, bool zin, Epilogue ep, const RhsArgs& a, hipStream_t s)
{
    if (zin && !a.virt && t.n_virt > 0) return hipErrorInvalidValue;
    if (zin && ep == kRkFirst && a.in != a.u) return hipErrorInvalidValue;   // the first stage takes the state from its input tiles
    if (!zin) {
        switch (ep) {
        case kOutPadded: return launch_one<KIND, false, kOutPadded>(t, a, s);
        case kOutZipped: return launch_one<KIND, false, kOutZipped>(t, a, s);
        case kRkFirst: return launch_one<KIND, false, kRkFirst>(t, a, s);
        case kRkMiddle: return launch_one<KIND, false, kRkMiddle>(t, a, s);
        case kRkLast: return launch_one<KIND, false, kRkLast>(t, a, s);
        default: return hipErrorInvalidValue;
        }
    }
    switch (ep) {
    case kOutZipped: return launch_one<KIND, true, kOutZipped>(t, a, s);
    case kRkFirst: return launch_one<KIND, true, kRkFirst>(t, a, s);
    case kRkMiddle: return launch_one<KIND, true, kRkMiddle>(t, a, s);
    case kRkLast: return launch_one<KIND, true, kRkLast>(t, a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_unzip(const DeviceTree& t, int nvar, const double* zipped, const double* virt, double* padded, hipStream_t s)
{
    if (t.nb <= 0 || nvar <= 0) return hipSuccess;
    if (!virt && t.n_virt > 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_unzip, dim3((unsigned)(t.nb * (nvar < NXCD ? nvar : NXCD))), dim3(NTHREADS), 0, s, t, nvar, zipped, virt, padded);
    return hipGetLastError();
}

hipError_t launch_virtual(const DeviceTree& t, int nvar, const double* zipped, double* virt, hipStream_t s)
{
    if (t.n_virt <= 0 || nvar <= 0) return hipSuccess;
    const int per = 8 / (nvar < 8 ? nvar : 8);       // virtual blocks per workgroup, as in the kernel
    hipLaunchKernelGGL(k_virtual, dim3(grid_for_blocks((t.n_virt + per - 1) / per)), dim3(NTHREADS), 0, s, t, nvar, zipped, virt);
    return hipGetLastError();
}

hipError_t launch_virtual_centred(const DeviceTree& t, const int64_t* vlevel_start, int nvar, const double* zipped, double* virt,
                                   hipStream_t s)
{
    if (t.n_virt <= 0 || nvar <= 0) return hipSuccess;
    for (int l = 0; l < 20; ++l) {                   // coarsest level first: a level's virtual blocks read those of the level before
        const int64_t n = vlevel_start[l + 1] - vlevel_start[l];
        if (n <= 0) continue;
        hipLaunchKernelGGL(k_virtual_centred, dim3(grid_for_blocks(n)), dim3(NTHREADS), 0, s, t, t.vlist + vlevel_start[l], n, nvar,
                           zipped, virt);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_zip(const DeviceTree& t, int nvar, const double* padded, double* zipped, hipStream_t s)
{
    const int64_t n = t.nb * nvar;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_zip, dim3((unsigned)n), dim3(NTHREADS), 0, s, n, padded, zipped);
    return hipGetLastError();
}

hipError_t launch_rhs(const DeviceTree& t, ot_rhs_kind kind, bool in_zipped, Epilogue ep, const RhsArgs& args, hipStream_t s)
{
    if (t.nb <= 0) return hipSuccess;
    switch (kind) {
    case OT_RHS_DERIVS: return launch_kind<OT_RHS_DERIVS>(t, in_zipped, ep, args, s);
    case OT_RHS_WAVE: return launch_kind<OT_RHS_WAVE>(t, in_zipped, ep, args, s);
    case OT_RHS_BURGERS: return launch_kind<OT_RHS_BURGERS>(t, in_zipped, ep, args, s);
    case OT_RHS_SYN24: return launch_kind<OT_RHS_SYN24>(t, in_zipped, ep, args, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace octfd
