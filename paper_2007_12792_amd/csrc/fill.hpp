// The two halves of a tile fill: request the planned values from memory, store them to LDS.  Private to kernels.hip.
#pragma once
#include "tile.hpp"

namespace octfd {
namespace {

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
