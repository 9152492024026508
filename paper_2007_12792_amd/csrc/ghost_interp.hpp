// Ghost values that come from a coarser leaf, for the kernels that write padded blocks (unzip, unzip_centred):
// separable six-point interpolation of whole boxes staged in LDS, with the clamped and the centred stencil
// rule; and the two halves of a tile fill (request from memory, store to LDS).  Private to kernels.hip.
#pragma once
#include "tile.hpp"

namespace octfd {
namespace {

// q / d for the few divisors that occur here (3, 8, 11, 14 and their pairwise products), q < 65536
__device__ __forceinline__ uint32_t div_magic(uint32_t d) { return 0xffffffffu / d + 1u; }
__device__ __forceinline__ int div_by(int q, uint32_t magic) { return (int)__umulhi((uint32_t)q, magic); }

// Interpolation of the boxes of the padded block that come from coarser leaves (every such leaf
// covers one box; a coarser leaf spans 16 fine points per axis and never contains the block itself,
// so a box is 3 or 11 points wide per axis and at least one axis is 3 wide).
// The x, y and z passes run over the boxes of SEVERAL source leaves at once ("round"), their work
// items packed densely over the 512 threads: four workgroup barriers per round instead of per
// source, and all source leaves of a round are requested from memory together.
// Staging per round: region A holds the coarse leaves (512 each) and, after the x pass, the y-pass
// results; region B, behind it, holds the x-pass results.
// done by one thread per block, once: boxes from the packed region ranges, greedy rounds in list order.
// with_corners = false: the sources that cover only a corner of the padded block (last in the list) are
// left out; the right-hand-side kernels never read the corners.
__device__ void make_box_plan(BlockInfo& bi, bool with_corners)
{
    BoxPlan& bp = bi.box;
    int nr = 0, sumc = 0, sum1 = 0, sum2 = 0, sum3 = 0, ns = 0;
    const int limit = with_corners ? 8 : bi.cs[29];
    bp.rbeg[0] = 0;
    for (int s = 0; s < limit; ++s) {
        if (bi.cs[2 * s] < 0) break;
        const int pk = bi.cs[2 * s + 1];
        const int rxl = pk & 3, rxh = (pk >> 2) & 3, ryl = (pk >> 4) & 3, ryh = (pk >> 6) & 3, rzl = (pk >> 8) & 3, rzh = (pk >> 10) & 3;
        const int sx = rxl == 0 ? 0 : (rxl == 1 ? PAD : PAD + NPT), ex = rxh == 0 ? PAD : (rxh == 1 ? PAD + NPT : NP);
        const int sy = ryl == 0 ? 0 : (ryl == 1 ? PAD : PAD + NPT), ey = ryh == 0 ? PAD : (ryh == 1 ? PAD + NPT : NP);
        const int sz = rzl == 0 ? 0 : (rzl == 1 ? PAD : PAD + NPT), ez = rzh == 0 ? PAD : (rzh == 1 ? PAD + NPT : NP);
        const int nx = ex - sx, ny = ey - sy, nz = ez - sz;
        const int t1 = 64 * nx, t2 = NPT * ny * nx, t3 = nz * ny * nx;
        // does the source still fit into the current round?
        const int a_need = max(sumc + BLK, sum2 + t2);
        if (s > bp.rbeg[nr] && (s - bp.rbeg[nr] == ROUND_SRC || a_need + sum1 + t1 > SCRATCH)) {
            bp.n1[nr] = sum1; bp.n2[nr] = sum2; bp.n3[nr] = sum3; bp.bstart[nr] = max(sumc, sum2);
            ++nr;
            bp.rbeg[nr] = s;
            sumc = sum1 = sum2 = sum3 = 0;
        }
        bp.o1[s] = sum1; bp.o2[s] = sum2; bp.o3[s] = sum3;
        sumc += BLK; sum1 += t1; sum2 += t2; sum3 += t3;
        bp.mx[s] = div_magic(nx); bp.mpl[s] = div_magic(nx * ny);
        bp.sx[s] = sx; bp.nx[s] = nx; bp.sy[s] = sy; bp.ny[s] = ny; bp.sz[s] = sz; bp.nz[s] = nz;
        // fine coordinate of the box's first point inside the coarse leaf (aligned to 16 points)
        bp.fx0[s] = (NPT * bi.ax + sx + 16 - PAD) & 15;
        bp.fy0[s] = (NPT * bi.ay + sy + 16 - PAD) & 15;
        bp.fz0[s] = (NPT * bi.az + sz + 16 - PAD) & 15;
        ns = s + 1;
    }
    if (ns > 0) {
        bp.n1[nr] = sum1; bp.n2[nr] = sum2; bp.n3[nr] = sum3; bp.bstart[nr] = max(sumc, sum2);
        ++nr;
        bp.rbeg[nr] = ns;
    }
    bp.nround = nr;
    for (int q = 0; q < bi.cs[16]; ++q) {
        int s = 0;
        while (s < ns - 1 && bi.cs[2 * s] != bi.cs[18 + 2 * q]) ++s;
        bp.face_src[q] = s;
    }
}
// the largest single box (11 x 11 x 3 or 3) must fit: 968 + 704
static_assert(NPT * 121 + 64 * 11 <= SCRATCH && BLK + 64 * 11 <= SCRATCH, "interpolation staging");

// Uniform control flow; starts with a barrier (the staging area may still be in use) and ends
// without one.  base = one variable's zipped array.
__device__ __forceinline__ void interp_boxes(double* tile, double* scratch, const BlockInfo& bi,
                                             const double* __restrict__ base, int tid)
{
    const BoxPlan& bp = bi.box;
    double cv[ROUND_SRC];
    auto request = [&](int r) {                  // the source leaves of round r, one element per thread and leaf
        const int s0 = bp.rbeg[r], s1 = bp.rbeg[r + 1];
#pragma unroll
        for (int q = 0; q < ROUND_SRC; ++q)
            if (s0 + q < s1) cv[q] = ldg(base, ((uint32_t)bi.cs[2 * (s0 + q)] * BLK + tid) * 8u);
    };
    if (bp.nround > 0) request(0);
#pragma unroll 1
    for (int r = 0; r < bp.nround; ++r) {
        const int s0 = bp.rbeg[r], s1 = bp.rbeg[r + 1];
        double* A = scratch;
        double* B = scratch + bp.bstart[r];
        __syncthreads();                         // everybody is done with the staging area
#pragma unroll
        for (int q = 0; q < ROUND_SRC; ++q)
            if (s0 + q < s1) A[q * BLK + tid] = cv[q];
        __syncthreads();
        if (r + 1 < bp.nround) request(r + 1);   // in flight during the three sweeps of this round
        for (int q = tid; q < bp.n1[r]; q += NTHREADS) {             // x pass, item (source, row = cz*8 + cy, tx)
            int s = s0;
            while (s + 1 < s1 && q >= bp.o1[s + 1]) ++s;
            const int local = q - bp.o1[s], nx = bp.nx[s];
            const int row = div_by(local, bp.mx[s]), tx = local - row * nx;
            B[q] = interp_line(&A[(s - s0) * BLK + row * NPT], 1, bp.fx0[s] + tx, bi.lag);
        }
        __syncthreads();
        for (int q = tid; q < bp.n2[r]; q += NTHREADS) {             // y pass, item (source, cz, ty, tx)
            int s = s0;
            while (s + 1 < s1 && q >= bp.o2[s + 1]) ++s;
            const int local = q - bp.o2[s], nx = bp.nx[s], pl = nx * bp.ny[s];
            const int cz = div_by(local, bp.mpl[s]), rr = local - cz * pl, ty = div_by(rr, bp.mx[s]), tx = rr - ty * nx;
            A[q] = interp_line(&B[bp.o1[s] + cz * NPT * nx + tx], nx, bp.fy0[s] + ty, bi.lag);
        }
        __syncthreads();
        for (int q = tid; q < bp.n3[r]; q += NTHREADS) {             // z pass, item (source, tz, ty, tx), into the tile
            int s = s0;
            while (s + 1 < s1 && q >= bp.o3[s + 1]) ++s;
            const int local = q - bp.o3[s], nx = bp.nx[s], pl = nx * bp.ny[s];
            const int tz = div_by(local, bp.mpl[s]), rr = local - tz * pl, ty = div_by(rr, bp.mx[s]), tx = rr - ty * nx;
            tile[tidx(bp.sz[s] + tz, bp.sy[s] + ty, bp.sx[s] + tx)] = interp_line(&A[bp.o2[s] + rr], pl, bp.fz0[s] + tz, bi.lag);
        }
    }
}

// The same for the centred variant of the ghost rule: the source is the coarser leaf's PADDED block
// (cpad, 14^3, filled by an earlier launch), every odd fine coordinate f takes the centred stencil
// on coarse nodes c0-2 .. c0+3, c0 = f >> 1, which may reach into that leaf's ghost layers.
// A box is 3 or 11 fine points wide per axis and needs 7 or 11 coarse nodes there (clo .. chi), and
// at least one axis is 3 wide: the coarse sub-box and the x- and y-pass results take at most 847
// doubles each, and two of the three are alive at a time.
constexpr int CENTRED_STAGING = 2 * 847;
static_assert(CENTRED_STAGING <= SCRATCH, "centred interpolation staging");
__device__ __forceinline__ double centred_line(const double* v, int st, int f, int clo, const double* lag)
{
    const int c0 = f >> 1;
    if (!(f & 1)) return v[(c0 - clo) * st];
    const double* w = lag + 12;                                  // the centred row, r = 5/2
    const double* p = v + (c0 - 2 - clo) * st;
    double acc = w[0] * p[0];
    acc = fma(w[1], p[st], acc);
    acc = fma(w[2], p[2 * st], acc);
    acc = fma(w[3], p[3 * st], acc);
    acc = fma(w[4], p[4 * st], acc);
    acc = fma(w[5], p[5 * st], acc);
    return acc;
}
// One box and its coarse sub-box.  The interpolation is split in two so that the memory latency of
// the next box hides behind the sweeps of the current one: request() loads this thread's (at most
// two) elements of the sub-box into registers, run() stages them and does the x, y and z passes.
struct CentredBox {
    int sx, nx, sy, ny, sz, nz, fx0, fy0, fz0, clx, cly, clz, ncx, ncy, ncz;
    const double* cpad;

    __device__ __forceinline__ void set(const BlockInfo& bi, const double* cpad_, int sx_, int nx_, int sy_, int ny_, int sz_, int nz_)
    {
        cpad = cpad_; sx = sx_; nx = nx_; sy = sy_; ny = ny_; sz = sz_; nz = nz_;
        fx0 = (NPT * bi.ax + sx + 16 - PAD) & 15;
        fy0 = (NPT * bi.ay + sy + 16 - PAD) & 15;
        fz0 = (NPT * bi.az + sz + 16 - PAD) & 15;
        clx = (fx0 >> 1) - 2; ncx = ((fx0 + nx - 1) >> 1) + 3 - clx + 1;
        cly = (fy0 >> 1) - 2; ncy = ((fy0 + ny - 1) >> 1) + 3 - cly + 1;
        clz = (fz0 >> 1) - 2; ncz = ((fz0 + nz - 1) >> 1) + 3 - clz + 1;
    }
    __device__ __forceinline__ void request(double (&c)[2], int tid) const
    {
        const uint32_t mcx = div_magic(ncx), mcxy = div_magic(ncx * ncy);
        const int n = ncz * ncy * ncx;                           // at most 847
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int q = tid + m * NTHREADS;
            if (q < n) {
                const int cz = div_by(q, mcxy), r = q - cz * ncx * ncy, cy = div_by(r, mcx), cx = r - cy * ncx;
                c[m] = cpad[((clz + cz + PAD) * NP + (cly + cy + PAD)) * NP + (clx + cx + PAD)];
            }
        }
    }
    // stores the requested elements; the caller may issue the next request() between stage() and sweep()
    __device__ __forceinline__ void stage(double* scratch, const double (&c)[2], int tid) const
    {
        double* C = scratch + ncz * ncy * nx;                    // behind the x-pass results; reused by the y pass
        const int n = ncz * ncy * ncx;
        __syncthreads();                                         // everybody is done with the staging arrays
#pragma unroll
        for (int m = 0; m < 2; ++m)
            if (tid + m * NTHREADS < n) C[tid + m * NTHREADS] = c[m];
        __syncthreads();
    }
    __device__ __forceinline__ void sweep(double* tile, double* scratch, const BlockInfo& bi, int tid) const
    {
        double* T1 = scratch;                    // after the x pass  [cz][cy][tx]
        double* T2 = T1 + ncz * ncy * nx;        // after the y pass  [cz][ty][tx]
        const double* C = T2;                    // the coarse sub-box [cz][cy][cx]: dead once the x pass is done
        const uint32_t mx = div_magic(nx), mxy = div_magic(nx * ny);
        for (int q = tid; q < ncz * ncy * nx; q += NTHREADS) {       // x pass, item (row = cz*ncy + cy, tx)
            const int row = div_by(q, mx), tx = q - row * nx;
            T1[q] = centred_line(&C[row * ncx], 1, fx0 + tx, clx, bi.lag);
        }
        __syncthreads();
        for (int q = tid; q < ncz * ny * nx; q += NTHREADS) {        // y pass, item (cz, ty, tx)
            const int cz = div_by(q, mxy), r = q - cz * nx * ny, ty = div_by(r, mx), tx = r - ty * nx;
            T2[q] = centred_line(&T1[cz * ncy * nx + tx], nx, fy0 + ty, cly, bi.lag);
        }
        __syncthreads();
        for (int q = tid; q < nz * ny * nx; q += NTHREADS) {         // z pass, into the tile
            const int tz = div_by(q, mxy), r = q - tz * nx * ny, ty = div_by(r, mx), tx = r - ty * nx;
            tile[tidx(sz + tz, sy + ty, sx + tx)] = centred_line(&T2[r], nx * ny, fz0 + tz, clz, bi.lag);
        }
    }
};

// every coarser source leaf of the block, one after the other; pbase = one variable's padded array of all blocks
__device__ __forceinline__ void interp_boxes_centred(double* tile, double* scratch, const BlockInfo& bi,
                                                     const double* __restrict__ pbase, int tid)
{
    const BoxPlan& bp = bi.box;
    const int ns = bp.rbeg[bp.nround];
    auto box = [&](CentredBox& cb, int s) {
        cb.set(bi, pbase + (int64_t)bi.cs[2 * s] * PBLK, bp.sx[s], bp.nx[s], bp.sy[s], bp.ny[s], bp.sz[s], bp.nz[s]);
    };
    if (ns == 0) return;
    CentredBox cur, nxt;
    double c[2];
    box(cur, 0);
    cur.request(c, tid);
#pragma unroll 1
    for (int s = 0; s < ns; ++s) {
        cur.stage(scratch, c, tid);
        if (s + 1 < ns) { box(nxt, s + 1); nxt.request(c, tid); }
        cur.sweep(tile, scratch, bi, tid);
        cur = nxt;
    }
}
// Filling the tile of one variable is split in two so that the global loads of the next variable
// can be in flight while the current one is being differentiated:
//   prefetch():   issue the planned loads into registers;
//   store_tile(): store them into a tile buffer.
// `base` is that variable's zipped array or this block's padded data.  All threads call both.
// USE = how many plan entries per thread are in use (PLAN_FACE: faces only).
// VIRT: plan entries with bit 0 set are offsets into vbase, that variable's virtual blocks.
template <int NPLAN, int USE, bool VIRT = false, bool REG>
__device__ __forceinline__ void prefetch(double (&v)[NPLAN], const FillPlan<NPLAN, REG>& fp, const double* __restrict__ base, int tid,
                                         const double* __restrict__ vbase = nullptr)
{
    uint32_t off[USE];
#pragma unroll
    for (int m = 0; m < USE; ++m) off[m] = fp.get_src(m, tid);
    // the last entry in use may reach beyond the face prefix: read element 0 instead
    if (USE == PLAN_FACE && NPLAN > PLAN_FACE && tid + (USE - 1) * NTHREADS >= NFACE) off[USE - 1] = 0;
#pragma unroll
    for (int m = 0; m < USE; ++m) {
        if (VIRT) v[m] = ldg((off[m] & 1u) ? vbase : base, off[m] & ~1u);
        else v[m] = ldg(base, off[m]);
    }
}

// the requested values into a tile buffer; does NOT end with a barrier
template <int NPLAN, int USE, bool REG>
__device__ __forceinline__ void store_tile(double* tile, const FillPlan<NPLAN, REG>& fp, const double (&v)[NPLAN], int tid)
{
#pragma unroll
    for (int m = 0; m < USE; ++m) {
        int d = fp.dst(m);
        if (USE == PLAN_FACE && NPLAN > PLAN_FACE && m == USE - 1 && tid + m * NTHREADS >= NFACE) d = DUMMY;
        tile[d] = v[m];
    }
}

}  // namespace
}  // namespace octfd
