// The 24-field synthetic system (see octfd.h, rhs_eval): what one pass over one variable computes at a thread's
// point, and the order in which the variables are streamed.  Shared by the one-block and the two-block kernels.
#pragma once
#include "stencils.hpp"

namespace octfd {
namespace {

// One SYN24 variable at this thread's point, fused axis by axis so that few values are live at any
// time (the scheduling fences keep the compiler from fetching every tap up front).  (nx, ny, nz)
// holds the gradient of the successor variable on entry and this variable's own gradient on exit.
//   t1 = beta . grad u,  t3q = grad u . grad u_next (before the factor 1/4),  ko = dissipation,
//   diag = Gxx Dxx + Gyy Dyy + Gzz Dzz (WITH_D2 only).
// WITH_D2 also publishes D1_y u and D1_z u of the own point for mixed_derivs().
struct Syn24Part { double t1, t3q, ko, diag; };

// SY, SZ: row and plane stride of the tile (and of the D1_z array)
template <bool WITH_D2, int SY = RS, int SZ = PS>
__device__ __forceinline__ Syn24Part syn24_axes(const double* t, int c, double* wy, double* wz, int owny, int ownz,
                                                double& nx, double& ny, double& nz, double bx, double by, double bz,
                                                double Gxx, double Gyy, double Gzz, double sigma, double ih, double ih2)
{
    Syn24Part r;
    const double u0 = t[c];
    r.diag = 0.0;
    const AxisOps x = axis_ops<WITH_D2>(t, c, 1, u0, ih, ih2);
    r.t1 = bx * x.d1;
    r.t3q = x.d1 * nx;
    nx = x.d1;
    if (WITH_D2) r.diag = Gxx * x.d2;
    double ksum = x.ko;
    __builtin_amdgcn_sched_barrier(0);
    const AxisOps y = axis_ops<WITH_D2>(t, c, SY, u0, ih, ih2);
    r.t1 = fma(by, y.d1, r.t1);
    r.t3q = fma(y.d1, ny, r.t3q);
    ny = y.d1;
    if (WITH_D2) { r.diag = fma(Gyy, y.d2, r.diag); wy[owny] = y.d1; }
    ksum = ksum + y.ko;
    __builtin_amdgcn_sched_barrier(0);
    const AxisOps z = axis_ops<WITH_D2>(t, c, SZ, u0, ih, ih2);
    r.t1 = fma(bz, z.d1, r.t1);
    r.t3q = fma(z.d1, nz, r.t3q);
    nz = z.d1;
    if (WITH_D2) { r.diag = fma(Gzz, z.d2, r.diag); wz[ownz] = z.d1; }
    r.ko = sigma * ((ksum + z.ko) * over64(ih));
    __builtin_amdgcn_sched_barrier(0);
    return r;
}

__device__ __forceinline__ double syn24_combine(const Syn24Part& p, int f, double lap, double halpha, double unext)
{
    const double kappa = __longlong_as_double((long long)(1023 - (f & 3)) << 52);   // 2^-(f mod 4)
    const double t2 = kappa * lap;
    const double t3 = 0.25 * p.t3q;
    const double t4 = halpha * unext;
    return (((p.t1 + t2) + t3) - t4) + p.ko;
}

// position t = 0..24 of the SYN24 variable stream -> variable.  Output a needs the gradient of
// variable a+1 (cyclically), so the variables are visited in descending cyclic order starting at 9:
// one gradient-only pass over variable 10, then 9, 8, ..., 0, 23, 22, ..., 10.  Every pass leaves
// its own gradient behind for the next one.
constexpr int NSTREAM = 25;
__device__ __forceinline__ int syn24_stream(int t) { return t == 0 ? 10 : (t <= 10 ? 10 - t : 34 - t); }

}  // namespace
}  // namespace octfd
