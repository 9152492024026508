// Clamped six-point Lagrange interpolation inside one coarse leaf (see octfd.h, unzip): shared by
// the ghost-fill kernels and the inter-grid transfer kernel so that both issue the same IEEE
// operation sequence.
#pragma once
#include <hip/hip_runtime.h>

namespace octfd {

// six-point Lagrange weights on nodes 0..5 at r = 1/2, 3/2, ..., 11/2 (numerators over 256)
static __constant__ double c_lag[36] = {
    63.0 / 256,  315.0 / 256, -210.0 / 256, 126.0 / 256,  -45.0 / 256,   7.0 / 256,
    -7.0 / 256,  105.0 / 256,  210.0 / 256, -70.0 / 256,   21.0 / 256,  -3.0 / 256,
     3.0 / 256,  -25.0 / 256,  150.0 / 256, 150.0 / 256,  -25.0 / 256,   3.0 / 256,
    -3.0 / 256,   21.0 / 256,  -70.0 / 256, 210.0 / 256,  105.0 / 256,  -7.0 / 256,
     7.0 / 256,  -45.0 / 256,  126.0 / 256, -210.0 / 256, 315.0 / 256,  63.0 / 256,
   -63.0 / 256,  385.0 / 256, -990.0 / 256, 1386.0 / 256, -1155.0 / 256, 693.0 / 256};

// 1-D interpolation inside a coarse leaf: v[0..7] (stride st) are its nodes, f in [0,16) the fine
// coordinate, lag a copy of c_lag.  Even f passes through; odd f uses the clamped six-node stencil.
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

}  // namespace octfd
