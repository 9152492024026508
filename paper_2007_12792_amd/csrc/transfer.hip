// gfx950 kernel of the inter-grid transfer (see octfd.h, regrid_transfer).  One workgroup of 512
// threads per target block, one thread per point, all variables in a loop.  What a block does is
// uniform over the workgroup: copy one source block, interpolate one octant of a coarser source
// block (x, y, z passes through LDS), or gather coinciding nodes from finer source blocks, each
// thread finding its source leaf by bisection over the Morton keys of the block's source run.
#include "lagrange.hpp"
#include "transfer.hpp"

namespace octfd {
namespace {

constexpr int NPT = 8, BLK = 512, NTHREADS = 512;

// spread the low 20 bits of v to every third bit
__device__ __forceinline__ uint64_t spread3(uint32_t v)
{
    uint64_t x = v & 0xfffffu;
    x = (x | (x << 32)) & 0x001f00000000ffffull;
    x = (x | (x << 16)) & 0x001f0000ff0000ffull;
    x = (x | (x << 8)) & 0x100f00f00f00f00full;
    x = (x | (x << 4)) & 0x10c30c30c30c30c3ull;
    x = (x | (x << 2)) & 0x1249249249249249ull;
    return x;
}

__global__ __launch_bounds__(NTHREADS) void k_transfer(DeviceTransfer t, int nvar, const double* __restrict__ in,
                                                       double* __restrict__ out)
{
    __shared__ double C[BLK], T1[BLK], T2[BLK], lag[36];
    const int tid = threadIdx.x;
    const int64_t b = blockIdx.x;
    const int i = tid & 7, j = (tid >> 3) & 7, k = tid >> 6;      // tid is also the point's index in its block
    const int32_t* row = t.table + b * kTransferRow;
    const int kind = row[0];
    const int64_t first = row[1];
    const size_t in_stride = static_cast<size_t>(t.n_from) * BLK, out_stride = static_cast<size_t>(t.n_to) * BLK;
    double* o = out + static_cast<size_t>(b) * BLK + tid;
    if (kind == kCopy) {
        const double* s = in + static_cast<size_t>(first) * BLK + tid;
        for (int v = 0; v < nvar; ++v) o[v * out_stride] = s[v * in_stride];
    } else if (kind == kProlong) {
        if (tid < 36) lag[tid] = c_lag[tid];
        const int oct = row[3];
        const int fx = NPT * (oct & 1) + i, fy = NPT * ((oct >> 1) & 1) + j, fz = NPT * ((oct >> 2) & 1) + k;
        const double* s = in + static_cast<size_t>(first) * BLK + tid;
        for (int v = 0; v < nvar; ++v) {
            __syncthreads();                                   // previous variable's passes are done
            C[tid] = s[v * in_stride];
            __syncthreads();
            T1[tid] = interp_line(&C[(k * NPT + j) * NPT], 1, fx, lag);           // (cz, cy, tx)
            __syncthreads();
            T2[tid] = interp_line(&T1[k * NPT * NPT + i], NPT, fy, lag);          // (cz, ty, tx)
            __syncthreads();
            o[v * out_stride] = interp_line(&T2[j * NPT + i], NPT * NPT, fz, lag);   // (tz, ty, tx)
        }
    } else {
        // the point is the lower corner of cell P of depth l+3; every source leaf is coarser than depth 20
        const ot_leaf T = t.to[b];
        const uint32_t l = T.level;
        const uint32_t px = NPT * T.ix + i, py = NPT * T.iy + j, pz = NPT * T.iz + k;
        const uint64_t key = l <= 17 ? (spread3(px << (17 - l)) | (spread3(py << (17 - l)) << 1) | (spread3(pz << (17 - l)) << 2))
                                     : (spread3(px >> (l - 17)) | (spread3(py >> (l - 17)) << 1) | (spread3(pz >> (l - 17)) << 2));
        int64_t lo = first, hi = first + row[2];               // last leaf of [lo, hi) whose key is <= key
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (t.from_keys[mid] <= key) lo = mid; else hi = mid;
        }
        const ot_leaf S = t.from[lo];
        const uint32_t d = S.level - l;                        // >= 1
        const uint32_t qx = (px << d) - NPT * S.ix, qy = (py << d) - NPT * S.iy, qz = (pz << d) - NPT * S.iz;
        const bool ok = qx < NPT && qy < NPT && qz < NPT;      // always true for a valid plan
        const double* s = in + static_cast<size_t>(lo) * BLK + (ok ? (qz * NPT + qy) * NPT + qx : 0);
        for (int v = 0; v < nvar; ++v) o[v * out_stride] = s[v * in_stride];
    }
}

}  // namespace

hipError_t launch_transfer(const DeviceTransfer& t, int nvar, const double* from_zipped, double* to_zipped,
                           hipStream_t s)
{
    if (t.n_to <= 0 || t.n_to > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_transfer, dim3(static_cast<unsigned>(t.n_to)), dim3(NTHREADS), 0, s, t, nvar, from_zipped, to_zipped);
    return hipGetLastError();
}

}  // namespace octfd
