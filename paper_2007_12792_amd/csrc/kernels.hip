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
#include "kernels.hpp"

namespace octfd {
namespace {

constexpr int NPT = 8, PAD = 3, NP = 14, BLK = 512, PBLK = 2744;
constexpr int NTHREADS = 512;
constexpr int K_COARSER = 2, K_SAME = 0;

// LDS geometry (in doubles).  Row stride 16 and plane stride 8 (mod 32) make the eight x-contiguous
// values of the four (j,k) pairs held by one half-wavefront fall into 32 different 8-byte banks.
constexpr int RS = 16;
constexpr int PS = NP * RS + 8;          // 232
constexpr int TILE = NP * PS;            // 14 planes
constexpr int WZ = NPT * PS;             // D1_z u on [8 k][14 jj][14 ii]
constexpr int YPS = NPT * RS + 8;        // plane stride of the D1_y array, 136
constexpr int WY = NPT * YPS;            // D1_y u on [8 k][8 j][14 ii]
constexpr int T1N = 64 * NP, T2N = NPT * NP * NP;            // interpolation staging
constexpr int SCRATCH = (WZ + WY) > (BLK + T1N + T2N) ? (WZ + WY) : (BLK + T1N + T2N);

// six-point Lagrange weights on nodes 0..5 at r = 1/2, 3/2, ..., 11/2 (numerators over 256)
__constant__ double c_lag[36] = {
    63.0 / 256,  315.0 / 256, -210.0 / 256, 126.0 / 256,  -45.0 / 256,   7.0 / 256,
    -7.0 / 256,  105.0 / 256,  210.0 / 256, -70.0 / 256,   21.0 / 256,  -3.0 / 256,
     3.0 / 256,  -25.0 / 256,  150.0 / 256, 150.0 / 256,  -25.0 / 256,   3.0 / 256,
    -3.0 / 256,   21.0 / 256,  -70.0 / 256, 210.0 / 256,  105.0 / 256,  -7.0 / 256,
     7.0 / 256,  -45.0 / 256,  126.0 / 256, -210.0 / 256, 315.0 / 256,  63.0 / 256,
   -63.0 / 256,  385.0 / 256, -990.0 / 256, 1386.0 / 256, -1155.0 / 256, 693.0 / 256};

struct BlockInfo {       // per-workgroup copy of the block's table rows
    int32_t gt[27 * 5];
    int32_t cs[16];      // coarse sources: {leaf id, packed region range} x 8, id < 0 ends the list
    uint32_t level, ax, ay, az;
    double lag[36];
};

__device__ __forceinline__ int tidx(int kk, int jj, int ii) { return kk * PS + jj * RS + ii; }

// thread -> interior point.  Lane bits 0-2 = i, bit 3 = j0, bit 4 = k0, bit 5 = j1; the wavefront
// number supplies j2 and k1, k2.  A half-wavefront thus covers 8 x 2 x 2 points.
__device__ __forceinline__ void point_of(int tid, int& i, int& j, int& k)
{
    const int w = tid >> 6;
    i = tid & 7;
    j = ((tid >> 3) & 1) | (((tid >> 5) & 1) << 1) | ((w & 1) << 2);
    k = ((tid >> 4) & 1) | ((w >> 1) << 1);
}

__device__ __forceinline__ void load_block_info(BlockInfo& bi, const DeviceTree& tr, int64_t b, int tid)
{
    if (tid < 27 * 5) bi.gt[tid] = tr.ghost[b * (27 * 5) + tid];
    if (tid >= 192 && tid < 192 + 36) bi.lag[tid - 192] = c_lag[tid - 192];
    if (tid >= 256 && tid < 256 + 16) bi.cs[tid - 256] = tr.coarse[b * 16 + (tid - 256)];
    if (tid == 320) {
        const ot_leaf lf = tr.leaves[b];
        bi.level = lf.level; bi.ax = lf.ix; bi.ay = lf.iy; bi.az = lf.iz;
    }
}

// ---------------------------------------------------------------- fill plan

constexpr int PLAN = (PBLK + NTHREADS - 1) / NTHREADS;   // 6 tile entries per thread

struct FillPlan { int src[PLAN]; int dst[PLAN]; };        // src < 0: nothing to copy

// Source of every padded point this thread fills, as an offset into one variable's zipped array
// (same-level copy or injection from a finer leaf).  Points whose source is coarser are left to
// the interpolation passes.
__device__ __forceinline__ void make_plan_zipped(FillPlan& fp, const BlockInfo& bi, int tid)
{
#pragma unroll
    for (int m = 0; m < PLAN; ++m) {
        const int p = tid + m * NTHREADS;
        fp.src[m] = -1; fp.dst[m] = 0;
        if (p >= PBLK) continue;
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        fp.dst[m] = tidx(kk, jj, ii);
        const int rx = ii < PAD ? 0 : (ii < PAD + NPT ? 1 : 2);
        const int ry = jj < PAD ? 0 : (jj < PAD + NPT ? 1 : 2);
        const int rz = kk < PAD ? 0 : (kk < PAD + NPT ? 1 : 2);
        const int32_t* e = &bi.gt[(rz * 9 + ry * 3 + rx) * 5];
        const int kind = e[0];
        if (kind == K_COARSER) continue;
        // coordinates inside the neighbouring octant of the same level, 0..7
        const int lx = ii - PAD + (1 - rx) * NPT, ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
        if (kind == K_SAME) {
            fp.src[m] = e[1] * BLK + (lz * NPT + ly) * NPT + lx;
        } else {
            // which child holds the point: forced by the direction on non-free axes
            const int bx = rx == 1 ? (lx >> 2) : (rx == 0 ? 1 : 0);
            const int by = ry == 1 ? (ly >> 2) : (ry == 0 ? 1 : 0);
            const int bz = rz == 1 ? (lz >> 2) : (rz == 0 ? 1 : 0);
            int q = 0, sh = 0;
            if (rx == 1) { q |= bx << sh; ++sh; }
            if (ry == 1) { q |= by << sh; ++sh; }
            if (rz == 1) { q |= bz << sh; }
            fp.src[m] = e[1 + q] * BLK + ((2 * lz - NPT * bz) * NPT + (2 * ly - NPT * by)) * NPT + (2 * lx - NPT * bx);
        }
    }
}

__device__ __forceinline__ void make_plan_padded(FillPlan& fp, int tid)
{
#pragma unroll
    for (int m = 0; m < PLAN; ++m) {
        const int p = tid + m * NTHREADS;
        const bool ok = p < PBLK;
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        fp.src[m] = ok ? p : -1;
        fp.dst[m] = ok ? tidx(kk, jj, ii) : 0;
    }
}

// 1-D interpolation inside a coarse leaf: v[0..7] (stride st) are its nodes, f in [0,16) the fine
// coordinate.  Even f passes through; odd f uses the clamped six-node stencil.
__device__ __forceinline__ double interp_line(const double* v, int st, int f, const double* lag)
{
    if (!(f & 1)) return v[(f >> 1) * st];
    const int c0 = (f - 1) >> 1;
    const int s = min(max(c0 - 2, 0), 2);
    const double* w = lag + (c0 - s) * 6;
    const double* p = v + s * st;
    double acc = w[0] * p[0];
    acc = fma(w[1], p[st], acc);
    acc = fma(w[2], p[2 * st], acc);
    acc = fma(w[3], p[3 * st], acc);
    acc = fma(w[4], p[4 * st], acc);
    acc = fma(w[5], p[5 * st], acc);
    return acc;
}

// Fill the tile of one variable.  `base` is that variable's zipped array (ZIN) or this block's
// padded data.  All threads call this; it ends with a barrier.  `scratch` is SCRATCH doubles.
template <bool ZIN>
__device__ __forceinline__ void fill_tile(double* tile, double* scratch, const BlockInfo& bi, const FillPlan& fp,
                                          const double* __restrict__ base, int tid)
{
    double v[PLAN];
#pragma unroll
    for (int m = 0; m < PLAN; ++m) if (fp.src[m] >= 0) v[m] = base[fp.src[m]];
#pragma unroll
    for (int m = 0; m < PLAN; ++m) if (fp.src[m] >= 0) tile[fp.dst[m]] = v[m];
    if (ZIN) {
        // every coarser source leaf covers a box of the padded block; interpolate box by box,
        // x then y then z.  Control flow is uniform over the workgroup.
        double* C = scratch;             // the coarse leaf, 8^3
        double* T1 = C + BLK;            // after the x pass  [cz][cy][tx], row stride NP
        double* T2 = T1 + T1N;           // after the y pass  [cz][ty][tx]
        for (int sidx = 0; sidx < 8; ++sidx) {
            const int32_t id = bi.cs[2 * sidx];
            if (id < 0) break;
            const int pk = bi.cs[2 * sidx + 1];
            const int rxl = pk & 3, rxh = (pk >> 2) & 3, ryl = (pk >> 4) & 3, ryh = (pk >> 6) & 3, rzl = (pk >> 8) & 3, rzh = (pk >> 10) & 3;
            const int sx = rxl == 0 ? 0 : (rxl == 1 ? PAD : PAD + NPT), ex = rxh == 0 ? PAD : (rxh == 1 ? PAD + NPT : NP);
            const int sy = ryl == 0 ? 0 : (ryl == 1 ? PAD : PAD + NPT), ey = ryh == 0 ? PAD : (ryh == 1 ? PAD + NPT : NP);
            const int sz = rzl == 0 ? 0 : (rzl == 1 ? PAD : PAD + NPT), ez = rzh == 0 ? PAD : (rzh == 1 ? PAD + NPT : NP);
            const int nx = ex - sx, ny = ey - sy, nz = ez - sz;
            // fine coordinate of the box's first point inside the coarse leaf (aligned to 16 points)
            const int fx0 = (NPT * bi.ax + sx + 16 - PAD) & 15;
            const int fy0 = (NPT * bi.ay + sy + 16 - PAD) & 15;
            const int fz0 = (NPT * bi.az + sz + 16 - PAD) & 15;
            C[tid] = base[(int64_t)id * BLK + tid];
            __syncthreads();
            for (int q = tid; q < 64 * nx; q += NTHREADS) {              // x pass
                const int tx = q % nx, row = q / nx;                     // row = cz*8 + cy
                T1[row * NP + tx] = interp_line(&C[row * NPT], 1, fx0 + tx, bi.lag);
            }
            __syncthreads();
            for (int q = tid; q < NPT * ny * nx; q += NTHREADS) {        // y pass
                const int tx = q % nx, ty = (q / nx) % ny, cz = q / (nx * ny);
                T2[(cz * NP + ty) * NP + tx] = interp_line(&T1[cz * NPT * NP + tx], NP, fy0 + ty, bi.lag);
            }
            __syncthreads();
            for (int q = tid; q < nz * ny * nx; q += NTHREADS) {         // z pass, into the tile
                const int tx = q % nx, ty = (q / nx) % ny, tz = q / (nx * ny);
                tile[tidx(sz + tz, sy + ty, sx + tx)] = interp_line(&T2[ty * NP + tx], NP * NP, fz0 + tz, bi.lag);
            }
            // the next source may overwrite C at once (last read two barriers ago); T1 and T2 are
            // rewritten only after further barriers
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------- stencils on the LDS tile

constexpr double C60 = 0x1.1111111111111p-6;   // 1/60
constexpr double C180 = 0x1.6c16c16c16c17p-8;  // 1/180

__device__ __forceinline__ double d1_taps(double m3, double m2, double m1, double p1, double p2, double p3, double ih)
{
    const double d1 = p1 - m1, d2 = p2 - m2, d3 = p3 - m3;
    double t = fma(-9.0, d2, d3);
    t = fma(45.0, d1, t);
    return (t * C60) * ih;
}

__device__ __forceinline__ double d1_at(const double* t, int c, int st, double ih)
{
    return d1_taps(t[c - 3 * st], t[c - 2 * st], t[c - st], t[c + st], t[c + 2 * st], t[c + 3 * st], ih);
}

// all centred operators along one axis share the six taps
struct AxisOps { double d1, d2, ko; };

template <bool WITH_D2>
__device__ __forceinline__ AxisOps axis_ops(const double* t, int c, int st, double u0, double ih, double ih2)
{
    const double m3 = t[c - 3 * st], m2 = t[c - 2 * st], m1 = t[c - st];
    const double p1 = t[c + st], p2 = t[c + 2 * st], p3 = t[c + 3 * st];
    AxisOps r;
    r.d1 = d1_taps(m3, m2, m1, p1, p2, p3, ih);
    const double s1 = p1 + m1, s2 = p2 + m2, s3 = p3 + m3;
    double q = fma(-6.0, s2, s3);
    q = fma(15.0, s1, q);
    r.ko = fma(-20.0, u0, q);
    if (WITH_D2) {
        double w = 2.0 * s3;
        w = fma(-27.0, s2, w);
        w = fma(270.0, s1, w);
        w = fma(-490.0, u0, w);
        r.d2 = (w * C180) * ih2;
    } else {
        r.d2 = 0.0;
    }
    return r;
}

struct PointOps { double u0, dx, dy, dz, lap, ko, dxx, dyy, dzz; };

template <bool WITH_D2>
__device__ __forceinline__ PointOps point_ops(const double* t, int c, double sigma, double ih, double ih2)
{
    PointOps r;
    r.u0 = t[c];
    const AxisOps x = axis_ops<WITH_D2>(t, c, 1, r.u0, ih, ih2);
    const AxisOps y = axis_ops<WITH_D2>(t, c, RS, r.u0, ih, ih2);
    const AxisOps z = axis_ops<WITH_D2>(t, c, PS, r.u0, ih, ih2);
    r.dx = x.d1; r.dy = y.d1; r.dz = z.d1;
    r.dxx = x.d2; r.dyy = y.d2; r.dzz = z.d2;
    r.lap = (x.d2 + y.d2) + z.d2;
    r.ko = sigma * (((x.ko + y.ko) + z.ko) * (ih * 0.015625));
    return r;
}

struct Mixed { double dxy, dxz, dyz; };

// Mixed derivatives of the variable in `tile` at this thread's point (i, j, k):
//   dxy = D1_x(D1_y u), dxz = D1_x(D1_z u), dyz = D1_y(D1_z u).
// wy [8][8][14] and wz [8][14][14] receive D1_y u and D1_z u; dy, dz are this thread's own values.
// Contains one barrier; the arrays may be reused after the next barrier.
__device__ __forceinline__ Mixed mixed_derivs(const double* tile, double* wy, double* wz, int tid, int i, int j, int k,
                                              double dy, double dz, double ih)
{
    wy[k * YPS + j * RS + (i + PAD)] = dy;
    wz[k * PS + (j + PAD) * RS + (i + PAD)] = dz;
    // ghost positions: 3 sets of 6 x 64 entries
    //   set 0: D1_y u at (ii ghost, j, k)      -> wy
    //   set 1: D1_z u at (ii ghost, j, k)      -> wz
    //   set 2: D1_z u at (i, jj ghost, k)      -> wz
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        const int q = tid + m * NTHREADS;
        if (q >= 3 * 384) break;
        const int set = q / 384, r = q % 384;
        if (set == 2) {
            const int g = r >> 6, kk = (r >> 3) & 7, ii = r & 7;
            const int jj = g < 3 ? g : g + NPT;
            wz[kk * PS + jj * RS + (ii + PAD)] = d1_at(tile, tidx(kk + PAD, jj, ii + PAD), PS, ih);
        } else {
            const int g = r % 6, jk = r / 6, jj = jk & 7, kk = jk >> 3;
            const int ii = g < 3 ? g : g + NPT;
            const int c = tidx(kk + PAD, jj + PAD, ii);
            if (set == 0) wy[kk * YPS + jj * RS + ii] = d1_at(tile, c, RS, ih);
            else wz[kk * PS + (jj + PAD) * RS + ii] = d1_at(tile, c, PS, ih);
        }
    }
    __syncthreads();
    Mixed r;
    r.dxy = d1_at(wy, k * YPS + j * RS + (i + PAD), 1, ih);
    const int cz = k * PS + (j + PAD) * RS + (i + PAD);
    r.dxz = d1_at(wz, cz, 1, ih);
    r.dyz = d1_at(wz, cz, RS, ih);
    return r;
}

// ---------------------------------------------------------------- output

template <int EPI>
__device__ __forceinline__ void emit(const RhsArgs& a, int64_t nb, int w, int64_t b, int pz, int cpad, double k)
{
    if (EPI == kOutPadded) {
        a.out[((int64_t)w * nb + b) * PBLK + cpad] = k;
        return;
    }
    const int64_t o = ((int64_t)w * nb + b) * BLK + pz;
    if (EPI == kOutZipped) {
        a.out[o] = k;
    } else if (EPI == kRkFirst) {
        a.acc[o] = k;
        a.out[o] = fma(a.c, k, a.u[o]);
    } else if (EPI == kRkMiddle) {
        a.acc[o] = a.acc[o] + 2.0 * k;
        a.out[o] = fma(a.c, k, a.u[o]);
    } else {
        a.u[o] = fma(a.c, a.acc[o] + k, a.u[o]);
    }
}

// ---------------------------------------------------------------- right-hand-side kernel

struct Pending { double part, ko, t4, dx, dy, dz; };   // a SYN24 output waiting for the next field's gradient

__device__ __forceinline__ double syn24_finish(const Pending& p, double dxn, double dyn, double dzn)
{
    double t3 = p.dx * dxn;
    t3 = fma(p.dy, dyn, t3);
    t3 = fma(p.dz, dzn, t3);
    t3 = 0.25 * t3;
    return ((p.part + t3) - p.t4) + p.ko;
}

template <int KIND, bool ZIN, int EPI>
__global__ __launch_bounds__(NTHREADS) void k_rhs(DeviceTree tr, RhsArgs a)
{
    __shared__ double tile[TILE];
    __shared__ double scratch[(ZIN || KIND == OT_RHS_SYN24) ? SCRATCH : 1];
    __shared__ BlockInfo bi;

    const int tid = threadIdx.x;
    const int64_t b = blockIdx.x, nb = tr.nb;
    load_block_info(bi, tr, b, tid);
    __syncthreads();

    int i, j, k;
    point_of(tid, i, j, k);
    const int c = tidx(k + PAD, j + PAD, i + PAD);
    const int pz = (k * NPT + j) * NPT + i;                          // offset inside a zipped block
    const int cpad = ((k + PAD) * NP + (j + PAD)) * NP + (i + PAD);  // offset inside a padded block
    const double ih = (double)(NPT << bi.level), ih2 = ih * ih;
    const double sigma = a.sigma;

    FillPlan fp;
    if (ZIN) make_plan_zipped(fp, bi, tid);
    else make_plan_padded(fp, tid);

    auto stage = [&](int v) {   // bring variable v into the tile (barrier before and after)
        __syncthreads();
        fill_tile<ZIN>(tile, scratch, bi, fp, ZIN ? a.in + (int64_t)v * nb * BLK : a.in + ((int64_t)v * nb + b) * PBLK, tid);
    };
    auto centre = [&](int v) -> double {   // this thread's own value of variable v
        return ZIN ? a.in[((int64_t)v * nb + b) * BLK + pz] : a.in[((int64_t)v * nb + b) * PBLK + cpad];
    };

    if (KIND == OT_RHS_DERIVS) {
        stage(0);
        const PointOps p = point_ops<true>(tile, c, 0.0, ih, ih2);
        emit<EPI>(a, nb, 0, b, pz, cpad, p.dx);
        emit<EPI>(a, nb, 1, b, pz, cpad, p.dy);
        emit<EPI>(a, nb, 2, b, pz, cpad, p.dz);
        emit<EPI>(a, nb, 3, b, pz, cpad, p.lap);
    } else if (KIND == OT_RHS_WAVE) {
        stage(0);
        const PointOps pu = point_ops<true>(tile, c, sigma, ih, ih2);
        stage(1);
        const PointOps pp = point_ops<false>(tile, c, sigma, ih, ih2);
        emit<EPI>(a, nb, 0, b, pz, cpad, pp.u0 + pu.ko);
        emit<EPI>(a, nb, 1, b, pz, cpad, pu.lap + pp.ko);
    } else if (KIND == OT_RHS_BURGERS) {
        stage(0);
        const PointOps p = point_ops<false>(tile, c, sigma, ih, ih2);
        const double flux = p.u0 * p.dx;
        emit<EPI>(a, nb, 0, b, pz, cpad, p.ko - flux);
    } else {
        // SYN24.  Fields are streamed in the order s, s+10, s+20 for s = 0..9 so that the
        // second-derivative combination Lap_s is consumed at once by the (up to) three outputs
        // that use it; each output waits in a Pending slot for the gradient of the next field.
        double* wz = scratch;
        double* wy = scratch + WZ;
        const double alpha = centre(0), bx = centre(1), by = centre(2), bz = centre(3);
        const double Gxx = 1.0 - 0.125 * centre(4), Gxy = -(0.125 * centre(5)), Gxz = -(0.125 * centre(6));
        const double Gyy = 1.0 - 0.125 * centre(7), Gyz = -(0.125 * centre(8)), Gzz = 1.0 - 0.125 * centre(9);
        const double halpha = 0.5 * alpha;
        Pending P0, P1, P2;
        double g0x = 0, g0y = 0, g0z = 0, g10x = 0, g10y = 0, g10z = 0, g20x = 0, g20y = 0, g20z = 0;

        auto open_slot = [&](Pending& P, int f, const PointOps& p, double lap, double unext) {
            double t1 = bx * p.dx;
            t1 = fma(by, p.dy, t1);
            t1 = fma(bz, p.dz, t1);
            const double kappa = __longlong_as_double((long long)(1023 - (f & 3)) << 52);   // 2^-(f mod 4)
            P.part = t1 + kappa * lap;
            P.ko = p.ko;
            P.t4 = halpha * unext;
            P.dx = p.dx; P.dy = p.dy; P.dz = p.dz;
        };

#pragma unroll 1
        for (int s = 0; s < 10; ++s) {
            double lap;
            {
                const double unext = centre((s + 11) % 24);
                stage(s);
                const PointOps p = point_ops<true>(tile, c, sigma, ih, ih2);
                const Mixed mx = mixed_derivs(tile, wy, wz, tid, i, j, k, p.dy, p.dz, ih);
                double diag = Gxx * p.dxx;
                diag = fma(Gyy, p.dyy, diag);
                diag = fma(Gzz, p.dzz, diag);
                double off = Gxy * mx.dxy;
                off = fma(Gxz, mx.dxz, off);
                off = fma(Gyz, mx.dyz, off);
                lap = fma(2.0, off, diag);
                if (s > 0) emit<EPI>(a, nb, s - 1, b, pz, cpad, syn24_finish(P0, p.dx, p.dy, p.dz));
                else { g0x = p.dx; g0y = p.dy; g0z = p.dz; }
                open_slot(P0, s, p, lap, unext);
            }
            {
                const double unext = centre((s + 21) % 24);
                stage(s + 10);
                const PointOps p = point_ops<false>(tile, c, sigma, ih, ih2);
                if (s > 0) emit<EPI>(a, nb, s + 9, b, pz, cpad, syn24_finish(P1, p.dx, p.dy, p.dz));
                else { g10x = p.dx; g10y = p.dy; g10z = p.dz; }
                open_slot(P1, s + 10, p, lap, unext);
            }
            if (s < 4) {
                const double unext = centre((s + 31) % 24);
                stage(s + 20);
                const PointOps p = point_ops<false>(tile, c, sigma, ih, ih2);
                if (s > 0) emit<EPI>(a, nb, s + 19, b, pz, cpad, syn24_finish(P2, p.dx, p.dy, p.dz));
                else { g20x = p.dx; g20y = p.dy; g20z = p.dz; }
                open_slot(P2, s + 20, p, lap, unext);
            }
        }
        emit<EPI>(a, nb, 9, b, pz, cpad, syn24_finish(P0, g10x, g10y, g10z));
        emit<EPI>(a, nb, 19, b, pz, cpad, syn24_finish(P1, g20x, g20y, g20z));
        emit<EPI>(a, nb, 23, b, pz, cpad, syn24_finish(P2, g0x, g0y, g0z));
    }
}

// ---------------------------------------------------------------- unzip / zip kernels

__global__ __launch_bounds__(NTHREADS) void k_unzip(DeviceTree tr, const double* __restrict__ zipped, double* __restrict__ padded)
{
    __shared__ double tile[TILE];
    __shared__ double scratch[SCRATCH];
    __shared__ BlockInfo bi;
    const int tid = threadIdx.x;
    const int64_t b = blockIdx.x, v = blockIdx.y, nb = tr.nb;
    load_block_info(bi, tr, b, tid);
    __syncthreads();
    FillPlan fp;
    make_plan_zipped(fp, bi, tid);
    fill_tile<true>(tile, scratch, bi, fp, zipped + v * nb * BLK, tid);
    double* out = padded + (v * nb + b) * PBLK;
#pragma unroll
    for (int m = 0; m < PLAN; ++m) {
        const int p = tid + m * NTHREADS;
        if (p < PBLK) out[p] = tile[fp.dst[m]];
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
    hipLaunchKernelGGL((k_rhs<KIND, ZIN, EPI>), dim3((unsigned)t.nb), dim3(NTHREADS), 0, s, t, a);
    return hipGetLastError();
}

template <int KIND>
hipError_t launch_kind(const DeviceTree& t, bool zin, Epilogue ep, const RhsArgs& a, hipStream_t s)
{
    if (!zin) return ep == kOutPadded ? launch_one<KIND, false, kOutPadded>(t, a, s) : hipErrorInvalidValue;
    switch (ep) {
    case kOutZipped: return launch_one<KIND, true, kOutZipped>(t, a, s);
    case kRkFirst: return launch_one<KIND, true, kRkFirst>(t, a, s);
    case kRkMiddle: return launch_one<KIND, true, kRkMiddle>(t, a, s);
    case kRkLast: return launch_one<KIND, true, kRkLast>(t, a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_unzip(const DeviceTree& t, int nvar, const double* zipped, double* padded, hipStream_t s)
{
    if (t.nb <= 0 || nvar <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_unzip, dim3((unsigned)t.nb, (unsigned)nvar), dim3(NTHREADS), 0, s, t, zipped, padded);
    return hipGetLastError();
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
