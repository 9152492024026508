// Finite-difference operators on the LDS tile and the ways a right-hand side leaves the kernel
// (plain store or Runge-Kutta stage update).  Private to kernels.hip.
#pragma once
#include "tile.hpp"

namespace octfd {
namespace {

// ---------------------------------------------------------------- stencils on the LDS tile

// x / 64 for a normal x >= 2^-1016 (here: 1/h = 2^(l+3)), done on the exponent bits: the same value as x * 0.015625,
// but integer arithmetic, which stays in scalar registers when x is uniform over the workgroup
__device__ __forceinline__ double over64(double x) { return __longlong_as_double(__double_as_longlong(x) - (6LL << 52)); }

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

// The three axes are evaluated one after the other (the scheduling fences keep the compiler from
// fetching all 19 taps up front): fewer values are live at once, which is what lets two workgroups
// share a compute unit.
template <bool WITH_D2>
__device__ __forceinline__ PointOps point_ops(const double* t, int c, double sigma, double ih, double ih2)
{
    PointOps r;
    r.u0 = t[c];
    const AxisOps x = axis_ops<WITH_D2>(t, c, 1, r.u0, ih, ih2);
    r.dx = x.d1; r.dxx = x.d2;
    __builtin_amdgcn_sched_barrier(0);
    const AxisOps y = axis_ops<WITH_D2>(t, c, RS, r.u0, ih, ih2);
    r.dy = y.d1; r.dyy = y.d2;
    const double kxy = x.ko + y.ko, lxy = x.d2 + y.d2;
    __builtin_amdgcn_sched_barrier(0);
    const AxisOps z = axis_ops<WITH_D2>(t, c, PS, r.u0, ih, ih2);
    r.dz = z.d1; r.dzz = z.d2;
    r.lap = lxy + z.d2;
    r.ko = sigma * ((kxy + z.ko) * over64(ih));
    __builtin_amdgcn_sched_barrier(0);
    return r;
}

struct Mixed { double dxy, dxz, dyz; };

// Mixed derivatives of the variable in `tile` at this thread's point:
//   dxy = D1_x(D1_y u), dxz = D1_x(D1_z u), dyz = D1_y(D1_z u).
// wy [8][8][14] and wz [8][14][14] hold D1_y u and D1_z u; every thread has already stored the
// values of its own point (indices owny, ownz).  The 3-deep ghost positions are whole-wavefront
// tasks: wavefronts 0..5 each take one ghost x index (64 (j,k) columns, both operators),
// wavefronts 2..7 each take one ghost y index.  Contains one barrier; the arrays may be reused
// after the next barrier.
__device__ __forceinline__ Mixed mixed_derivs(const double* tile, double* wy, double* wz, int tid, int owny, int ownz, double ih)
{
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int la = tid & 7, lb = (tid >> 3) & 7;       // lane coordinates inside the task
    if (w < 6) {                                        // ghost x index ii, lanes = (j, k)
        const int ii = w < 3 ? w : w + NPT;
        const int ct = tidx(lb + PAD, la + PAD, ii);
        wy[lb * YPS + la * RS + ii] = d1_at(tile, ct, RS, ih);
        wz[lb * PS + (la + PAD) * RS + ii] = d1_at(tile, ct, PS, ih);
    }
    if (w >= 2) {                                       // ghost y index jj, lanes = (i, k)
        const int g = w - 2, jj = g < 3 ? g : g + NPT;
        const int ct = tidx(lb + PAD, jj, la + PAD);
        wz[lb * PS + jj * RS + (la + PAD)] = d1_at(tile, ct, PS, ih);
    }
    __syncthreads();
    Mixed r;
    r.dxy = d1_at(wy, owny, 1, ih);
    __builtin_amdgcn_sched_barrier(0);
    r.dxz = d1_at(wz, ownz, 1, ih);
    __builtin_amdgcn_sched_barrier(0);
    r.dyz = d1_at(wz, ownz, RS, ih);
    return r;
}

// ---------------------------------------------------------------- output

// The Runge-Kutta epilogues read the accumulator and the state at the thread's own point.  Those
// loads are issued at the start of a variable's pass (epi_prefetch) and consumed at its end (emit),
// so their latency hides behind the stencil work.
// o8 = byte offset of this thread's point inside one variable's zipped array, p8 = inside one
// padded block; w selects the variable and b the block (both uniform).
struct EpiOperands { double acc, u; };

// U_FROM_TILE: in the first stage the input of the right-hand side is the state itself (the launcher checks it), so
// the state at the thread's point is the centre of the variable's tile and is not loaded again: the kernel hands it
// over with with_u() once it has it.
template <int EPI, bool U_FROM_TILE = false>
__device__ __forceinline__ EpiOperands epi_prefetch(const RhsArgs& a, int64_t nb, int w, uint32_t o8)
{
    EpiOperands e{0.0, 0.0};
    const int64_t f = (int64_t)w * nb * BLK;
    if ((EPI == kRkFirst && !U_FROM_TILE) || EPI == kRkMiddle || EPI == kRkLast) e.u = ldg(a.u + f, o8);
    if (EPI == kRkMiddle || EPI == kRkLast) e.acc = ldg(a.acc + f, o8);
    return e;
}
template <int EPI>
__device__ __forceinline__ EpiOperands with_u(EpiOperands e, double centre)
{
    if (EPI == kRkFirst) e.u = centre;
    return e;
}

template <int EPI>
__device__ __forceinline__ void emit(const RhsArgs& a, int64_t nb, int w, int64_t b, uint32_t o8, uint32_t p8, double k,
                                     const EpiOperands& e)
{
    if (EPI == kOutPadded) {
        stg(a.out + ((int64_t)w * nb + b) * PBLK, p8, k);
        return;
    }
    const int64_t f = (int64_t)w * nb * BLK;
    if (EPI == kOutZipped) {
        stg(a.out + f, o8, k);
    } else if (EPI == kRkFirst) {
        stg(a.acc + f, o8, k);
        stg(a.out + f, o8, fma(a.c, k, e.u));
    } else if (EPI == kRkMiddle) {
        stg(a.acc + f, o8, e.acc + 2.0 * k);
        stg(a.out + f, o8, fma(a.c, k, e.u));
    } else {
        stg(a.u + f, o8, fma(a.c, e.acc + k, e.u));
    }
}

}  // namespace
}  // namespace octfd
