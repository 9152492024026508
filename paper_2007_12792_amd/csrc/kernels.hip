// gfx950 kernels of liboctfd.  One workgroup of 512 threads (8 wavefronts) owns one block; thread
// tid owns interior point (i, j, k) = (tid & 7, (tid >> 3) & 7, tid >> 6), so zipped loads and
// stores are contiguous.  A ghost-padded 14^3 tile of one variable lives in LDS; variables are
// streamed through it one at a time.  The tile is filled either from a padded array (plain copy)
// or straight from zipped storage through the ghost-source table (copy, injection, separable
// Lagrange interpolation staged in LDS), which is what `unzip` writes out and what the fused
// right-hand-side kernels consume without ever materialising the padded array.
//
// Arithmetic follows one fixed IEEE sequence per formula (see octfd.h); the file is compiled with
// -ffp-contract=off, so a fused multiply-add happens exactly where fma() is written.
#include "kernels.hpp"

namespace octfd {
namespace {

constexpr int NPT = 8, PAD = 3, NP = 14, BLK = 512, PBLK = 2744;
constexpr int NTHREADS = 512;
constexpr int RS = 14;            // LDS row stride of the tile, in doubles
constexpr int PS = NP * RS + 2;   // LDS plane stride
constexpr int TILE = NP * PS;
constexpr int K_SAME = 0, K_FINER = 1, K_COARSER = 2;

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
    uint32_t level, ax, ay, az;
    double lag[36];
};

struct FillScratch {     // staging for coarse-to-fine interpolation
    double C[BLK];       // the coarse source leaf
    double T1[BLK];      // after the x pass  [cz][cy][tx]
    double T2[BLK];      // after the y pass  [cz][ty][tx]
};

__device__ __forceinline__ int tidx(int kk, int jj, int ii) { return kk * PS + jj * RS + ii; }

__device__ __forceinline__ void load_block_info(BlockInfo& bi, const DeviceTree& tr, int64_t b, int tid)
{
    if (tid < 27 * 5) bi.gt[tid] = tr.ghost[b * (27 * 5) + tid];
    if (tid >= 192 && tid < 192 + 36) bi.lag[tid - 192] = c_lag[tid - 192];
    if (tid == 256) {
        const ot_leaf lf = tr.leaves[b];
        bi.level = lf.level; bi.ax = lf.ix; bi.ay = lf.iy; bi.az = lf.iz;
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

// Fill the LDS tile of one variable from zipped storage.  zvar = that variable's [nb][512] array.
// All threads of the workgroup must call this; it ends with a barrier.
__device__ void fill_tile(double* tile, FillScratch& fs, const BlockInfo& bi, const double* __restrict__ zvar, int tid)
{
    // phase A: copies from same-level leaves and injections from finer leaves
    for (int p = tid; p < PBLK; p += NTHREADS) {
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        const int rx = ii < PAD ? 0 : (ii < PAD + NPT ? 1 : 2);
        const int ry = jj < PAD ? 0 : (jj < PAD + NPT ? 1 : 2);
        const int rz = kk < PAD ? 0 : (kk < PAD + NPT ? 1 : 2);
        const int32_t* e = &bi.gt[(rz * 9 + ry * 3 + rx) * 5];
        const int kind = e[0];
        if (kind == K_COARSER) continue;
        // coordinates inside the neighbouring octant of the same level, 0..7
        const int lx = ii - PAD + (1 - rx) * NPT, ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
        int64_t src; int off;
        if (kind == K_SAME) {
            src = e[1];
            off = (lz * NPT + ly) * NPT + lx;
        } else {
            // which child holds the point: forced by the direction on non-free axes
            const int bx = rx == 1 ? (lx >> 2) : (rx == 0 ? 1 : 0);
            const int by = ry == 1 ? (ly >> 2) : (ry == 0 ? 1 : 0);
            const int bz = rz == 1 ? (lz >> 2) : (rz == 0 ? 1 : 0);
            int q = 0, sh = 0;
            if (rx == 1) { q |= bx << sh; ++sh; }
            if (ry == 1) { q |= by << sh; ++sh; }
            if (rz == 1) { q |= bz << sh; }
            src = e[1 + q];
            off = ((2 * lz - NPT * bz) * NPT + (2 * ly - NPT * by)) * NPT + (2 * lx - NPT * bx);
        }
        tile[tidx(kk, jj, ii)] = zvar[src * BLK + off];
    }
    // phase B: regions whose source leaf is coarser.  Control flow is uniform over the workgroup.
    int32_t staged = -1;
    for (int dir = 0; dir < 27; ++dir) {
        if (bi.gt[dir * 5] != K_COARSER) continue;
        const int32_t id = bi.gt[dir * 5 + 1];
        const int rx = dir % 3, ry = (dir / 3) % 3, rz = dir / 9;
        const int nx = rx == 1 ? NPT : PAD, ny = ry == 1 ? NPT : PAD, nz = rz == 1 ? NPT : PAD;
        // first padded index of the region, and first fine coordinate inside the coarse leaf
        const int sx = rx == 0 ? 0 : (rx == 1 ? PAD : PAD + NPT);
        const int sy = ry == 0 ? 0 : (ry == 1 ? PAD : PAD + NPT);
        const int sz = rz == 0 ? 0 : (rz == 1 ? PAD : PAD + NPT);
        const int fx0 = NPT * ((bi.ax + rx - 1) & 1) + (rx == 0 ? NPT - PAD : 0);
        const int fy0 = NPT * ((bi.ay + ry - 1) & 1) + (ry == 0 ? NPT - PAD : 0);
        const int fz0 = NPT * ((bi.az + rz - 1) & 1) + (rz == 0 ? NPT - PAD : 0);
        if (id != staged) {                        // C was last read two barriers ago
            fs.C[tid] = zvar[(int64_t)id * BLK + tid];
            staged = id;
        }
        __syncthreads();
        if (tid < 64 * nx) {                       // x pass
            const int tx = tid % nx, row = tid / nx;             // row = cz*8 + cy
            fs.T1[row * NPT + tx] = interp_line(&fs.C[row * NPT], 1, fx0 + tx, bi.lag);
        }
        __syncthreads();
        if (tid < NPT * ny * nx) {                 // y pass
            const int tx = tid % nx, ty = (tid / nx) % ny, cz = tid / (nx * ny);
            fs.T2[(cz * NPT + ty) * NPT + tx] = interp_line(&fs.T1[cz * 64 + tx], NPT, fy0 + ty, bi.lag);
        }
        __syncthreads();
        if (tid < nz * ny * nx) {                  // z pass, into the tile
            const int tx = tid % nx, ty = (tid / nx) % ny, tz = tid / (nx * ny);
            tile[tidx(sz + tz, sy + ty, sx + tx)] = interp_line(&fs.T2[ty * NPT + tx], 64, fz0 + tz, bi.lag);
        }
    }
    __syncthreads();
}

// plain copy of one padded block into the tile
__device__ __forceinline__ void copy_tile(double* tile, const double* __restrict__ pblock, int tid)
{
    for (int p = tid; p < PBLK; p += NTHREADS) {
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        tile[tidx(kk, jj, ii)] = pblock[p];
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

// mixed derivative D1 along stride sa of (D1 along stride sb)
__device__ __forceinline__ double dmix_at(const double* t, int c, int sa, int sb, double ih)
{
    return d1_taps(d1_at(t, c - 3 * sa, sb, ih), d1_at(t, c - 2 * sa, sb, ih), d1_at(t, c - sa, sb, ih),
                   d1_at(t, c + sa, sb, ih), d1_at(t, c + 2 * sa, sb, ih), d1_at(t, c + 3 * sa, sb, ih), ih);
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

// ---------------------------------------------------------------- output

template <int EPI>
__device__ __forceinline__ void emit(const RhsArgs& a, int64_t nb, int w, int64_t b, int tid, int cpad, double k)
{
    if (EPI == kOutPadded) {
        a.out[((int64_t)w * nb + b) * PBLK + cpad] = k;
        return;
    }
    const int64_t o = ((int64_t)w * nb + b) * BLK + tid;
    if (EPI == kOutZipped) {
        a.out[o] = k;
    } else if (EPI == kRkFirst) {
        a.acc[o] = k;
        a.out[o] = fma(a.c, k, a.in[o]);
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
    __shared__ BlockInfo bi;
    __shared__ double fs_raw[ZIN ? sizeof(FillScratch) / sizeof(double) : 1];   // staging only exists when filling from zipped data
    FillScratch& fs = *reinterpret_cast<FillScratch*>(fs_raw);

    const int tid = threadIdx.x;
    const int64_t b = blockIdx.x, nb = tr.nb;
    load_block_info(bi, tr, b, tid);
    __syncthreads();

    const int i = tid & 7, j = (tid >> 3) & 7, k = tid >> 6;
    const int c = tidx(k + PAD, j + PAD, i + PAD);
    const int cpad = ((k + PAD) * NP + (j + PAD)) * NP + (i + PAD);
    const double ih = (double)(NPT << bi.level), ih2 = ih * ih;
    const double sigma = a.sigma;

    auto stage = [&](int v) {   // bring variable v into the tile (barrier before and after)
        __syncthreads();
        if (ZIN) fill_tile(tile, fs, bi, a.in + (int64_t)v * nb * BLK, tid);
        else copy_tile(tile, a.in + ((int64_t)v * nb + b) * PBLK, tid);
    };
    auto centre = [&](int v) -> double {   // this thread's own value of variable v
        return ZIN ? a.in[((int64_t)v * nb + b) * BLK + tid] : a.in[((int64_t)v * nb + b) * PBLK + cpad];
    };

    if (KIND == OT_RHS_DERIVS) {
        stage(0);
        const PointOps p = point_ops<true>(tile, c, 0.0, ih, ih2);
        emit<EPI>(a, nb, 0, b, tid, cpad, p.dx);
        emit<EPI>(a, nb, 1, b, tid, cpad, p.dy);
        emit<EPI>(a, nb, 2, b, tid, cpad, p.dz);
        emit<EPI>(a, nb, 3, b, tid, cpad, p.lap);
    } else if (KIND == OT_RHS_WAVE) {
        stage(0);
        const PointOps pu = point_ops<true>(tile, c, sigma, ih, ih2);
        stage(1);
        const PointOps pp = point_ops<false>(tile, c, sigma, ih, ih2);
        emit<EPI>(a, nb, 0, b, tid, cpad, pp.u0 + pu.ko);
        emit<EPI>(a, nb, 1, b, tid, cpad, pu.lap + pp.ko);
    } else if (KIND == OT_RHS_BURGERS) {
        stage(0);
        const PointOps p = point_ops<false>(tile, c, sigma, ih, ih2);
        const double flux = p.u0 * p.dx;
        emit<EPI>(a, nb, 0, b, tid, cpad, p.ko - flux);
    } else {
        // SYN24.  Fields are streamed in the order s, s+10, s+20 for s = 0..9 so that the
        // second-derivative combination Lap_s is consumed at once by the (up to) three outputs
        // that use it; each output waits in a Pending slot for the gradient of the next field.
        const double alpha = centre(0), bx = centre(1), by = centre(2), bz = centre(3);
        const double Gxx = 1.0 - 0.125 * centre(4), Gxy = -(0.125 * centre(5)), Gxz = -(0.125 * centre(6));
        const double Gyy = 1.0 - 0.125 * centre(7), Gyz = -(0.125 * centre(8)), Gzz = 1.0 - 0.125 * centre(9);
        const double halpha = 0.5 * alpha;
        Pending P0, P1, P2;
        double g0x = 0, g0y = 0, g0z = 0, g10x = 0, g10y = 0, g10z = 0, g20x = 0, g20y = 0, g20z = 0;

        auto open_slot = [&](Pending& P, int f, const PointOps& p, double lap) {
            double t1 = bx * p.dx;
            t1 = fma(by, p.dy, t1);
            t1 = fma(bz, p.dz, t1);
            const double kappa = __longlong_as_double((long long)(1023 - (f & 3)) << 52);   // 2^-(f mod 4)
            P.part = t1 + kappa * lap;
            P.ko = p.ko;
            P.t4 = halpha * centre((f + 11) % 24);
            P.dx = p.dx; P.dy = p.dy; P.dz = p.dz;
        };

        for (int s = 0; s < 10; ++s) {
            double lap;
            {
                stage(s);
                const PointOps p = point_ops<true>(tile, c, sigma, ih, ih2);
                const double dxy = dmix_at(tile, c, 1, RS, ih);
                const double dxz = dmix_at(tile, c, 1, PS, ih);
                const double dyz = dmix_at(tile, c, RS, PS, ih);
                double diag = Gxx * p.dxx;
                diag = fma(Gyy, p.dyy, diag);
                diag = fma(Gzz, p.dzz, diag);
                double off = Gxy * dxy;
                off = fma(Gxz, dxz, off);
                off = fma(Gyz, dyz, off);
                lap = fma(2.0, off, diag);
                if (s > 0) emit<EPI>(a, nb, s - 1, b, tid, cpad, syn24_finish(P0, p.dx, p.dy, p.dz));
                else { g0x = p.dx; g0y = p.dy; g0z = p.dz; }
                open_slot(P0, s, p, lap);
            }
            {
                stage(s + 10);
                const PointOps p = point_ops<false>(tile, c, sigma, ih, ih2);
                if (s > 0) emit<EPI>(a, nb, s + 9, b, tid, cpad, syn24_finish(P1, p.dx, p.dy, p.dz));
                else { g10x = p.dx; g10y = p.dy; g10z = p.dz; }
                open_slot(P1, s + 10, p, lap);
            }
            if (s < 4) {
                stage(s + 20);
                const PointOps p = point_ops<false>(tile, c, sigma, ih, ih2);
                if (s > 0) emit<EPI>(a, nb, s + 19, b, tid, cpad, syn24_finish(P2, p.dx, p.dy, p.dz));
                else { g20x = p.dx; g20y = p.dy; g20z = p.dz; }
                open_slot(P2, s + 20, p, lap);
            }
        }
        emit<EPI>(a, nb, 9, b, tid, cpad, syn24_finish(P0, g10x, g10y, g10z));
        emit<EPI>(a, nb, 19, b, tid, cpad, syn24_finish(P1, g20x, g20y, g20z));
        emit<EPI>(a, nb, 23, b, tid, cpad, syn24_finish(P2, g0x, g0y, g0z));
    }
}

// ---------------------------------------------------------------- unzip / zip kernels

__global__ __launch_bounds__(NTHREADS) void k_unzip(DeviceTree tr, const double* __restrict__ zipped, double* __restrict__ padded)
{
    __shared__ double tile[TILE];
    __shared__ BlockInfo bi;
    __shared__ FillScratch fs;
    const int tid = threadIdx.x;
    const int64_t b = blockIdx.x, v = blockIdx.y, nb = tr.nb;
    load_block_info(bi, tr, b, tid);
    __syncthreads();
    fill_tile(tile, fs, bi, zipped + v * nb * BLK, tid);
    double* out = padded + (v * nb + b) * PBLK;
    for (int p = tid; p < PBLK; p += NTHREADS) {
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        out[p] = tile[tidx(kk, jj, ii)];
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
