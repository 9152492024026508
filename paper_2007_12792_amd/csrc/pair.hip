// gfx950 kernel of the 24-field right-hand side on zipped input: TWO sibling blocks per workgroup.
//
// Two leaves that are x-neighbours inside one parent follow each other in storage.  One workgroup of
// 1,024 threads (16 wavefronts, one whole compute unit) owns such a pair as a single 16 x 8 x 8 brick with a
// 22 x 14 x 14 tile: the face between the two blocks is interior, so none of its 2 x 3 x 64 ghost points is
// fetched, and the two x faces that remain are the expensive ones (an x ghost uses 3 of the 8 values of a row,
// so an x face costs the neighbour's whole 4 KB).  Ghost points per point fall from 3.94 to 3.0.
//
// With the compute unit's 160 KB of LDS to itself the workgroup also keeps the ten second-derivative
// combinations Lap_s of its points in LDS (80 KB) instead of parking them in memory, which the one-block
// kernel must do.  The tile is single-buffered: data of the next variable waits in registers until every
// thread has finished with the tile.
//
// Everything a thread computes at its point is the same IEEE sequence as in the one-block kernel
// (stencils.hpp, syn24.hpp); only where the operands sit in LDS differs.  Ghost values that would come from a
// coarser leaf are read from virtual blocks (see HostTree), so no interpolation happens here.
#include "kernels.hpp"
#include "stencils.hpp"
#include "syn24.hpp"
#include "tile.hpp"

#include <type_traits>

namespace octfd {
namespace {

namespace pr {
constexpr int NT = 1024;
constexpr int NX = 2 * NPT + 2 * PAD;    // 22 tile points along x
constexpr int RS = NX;                   // row stride
constexpr int PS = NX * NP + 4;          // plane stride 312 = 24 (mod 32): eight x-contiguous values of four k planes
                                         // fall into 32 different 8-byte banks, as in the one-block tile
constexpr int TILE = NP * PS;            // 14 planes
constexpr int WZ = NPT * PS;             // D1_z u on [8 k][14 jj][22 ii], rows and planes strided like the tile
constexpr int YPS = NPT * RS + 8;        // 184 = 24 (mod 32)
constexpr int WY = NPT * YPS;            // D1_y u on [8 k][8 j][22 ii]
constexpr int DUMMY = NX * NP;           // first padding slot behind plane 0: where masked plan entries are stored
// ghost points of the tile in the order they are planned: the faces, then the edges (corners are never read)
constexpr int NGF = 2 * PAD * NPT * NPT + 4 * PAD * 2 * NPT * NPT;                  // 1920
constexpr int NGE = NGF + 8 * PAD * PAD * NPT + 4 * PAD * PAD * 2 * NPT;           // 3072 = 3 * NT
constexpr int USE_FACE = 2, USE_EDGE = 3;                                          // plan entries per thread in use
static_assert(NGE == 3 * NT && NGF <= 2 * NT, "plan entries per thread");
constexpr int PAIR_CHUNK = 32;           // pairs per chunk: the 32 workgroups that run on an XCD at a time take 64 consecutive blocks
                                         // (measured on the 102,075-block tree: 59.6 / 58.8 / 58.3 / 57.9 / 57.8 ms per step for 1 / 4 / 8 / 16 / 32)

__device__ __forceinline__ int gx(int g) { return g < PAD ? g : g + 2 * NPT; }     // 0,1,2,19,20,21
__device__ __forceinline__ int gyz(int g) { return g < PAD ? g : g + NPT; }        // 0,1,2,11,12,13

// p-th ghost point of the tile
__device__ __forceinline__ void ghost_point(int p, int& ii, int& jj, int& kk)
{
    if (p < 384) {                                   // x faces: 6 ghosts of each of the 64 interior rows
        const int r = p / 6;
        ii = gx(p - 6 * r); jj = PAD + (r & 7); kk = PAD + (r >> 3);
    } else if (p < 384 + 768) {                      // y faces
        const int q = p - 384, r = q >> 4, kq = r / 6;
        ii = PAD + (q & 15); jj = gyz(r - 6 * kq); kk = PAD + kq;
    } else if (p < NGF) {                            // z faces
        const int q = p - (384 + 768);
        ii = PAD + (q & 15); jj = PAD + ((q >> 4) & 7); kk = gyz(q >> 7);
    } else if (p < NGF + 288) {                      // xy edges
        const int q = p - NGF, r = q / 6, kq = r / 6;
        ii = gx(q - 6 * r); jj = gyz(r - 6 * kq); kk = PAD + kq;
    } else if (p < NGF + 576) {                      // xz edges
        const int q = p - (NGF + 288), r = q / 6;
        ii = gx(q - 6 * r); jj = PAD + (r & 7); kk = gyz(r >> 3);
    } else {                                         // yz edges
        const int q = p - (NGF + 576), r = q >> 4, kg = r / 6;
        ii = PAD + (q & 15); jj = gyz(r - 6 * kg); kk = gyz(kg);
    }
}

// Mixed derivatives at the thread's point, as mixed_derivs() of the one-block kernel: every thread has stored
// D1_y u and D1_z u of its own point; the 3-deep ghost positions are whole-wavefront tasks (wavefronts 0..5: one ghost
// x column each, both operators; wavefronts 4..15: half a ghost y row each).  fill() ends before the barrier that
// the caller places; taps() follows it.
__device__ __forceinline__ void mixed_fill(const double* tile, double* wy, double* wz, int tid, double ih)
{
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int la = tid & 7, lb = (tid >> 3) & 7;
    if (w < 6) {                                     // ghost x index ii, lanes = (j, k)
        const int ii = gx(w);
        const int ct = (lb + PAD) * PS + (la + PAD) * RS + ii;
        wy[lb * YPS + la * RS + ii] = d1_at(tile, ct, RS, ih);
        wz[lb * PS + (la + PAD) * RS + ii] = d1_at(tile, ct, PS, ih);
    }
    if (w >= 4) {                                    // ghost y index jj of one of the two blocks, lanes = (i, k)
        const int g = w - 4, jj = gyz(g >> 1), ix = la + PAD + NPT * (g & 1);
        wz[lb * PS + jj * RS + ix] = d1_at(tile, (lb + PAD) * PS + jj * RS + ix, PS, ih);
    }
}
__device__ __forceinline__ Mixed mixed_taps(const double* wy, const double* wz, int owny, int ownz, double ih)
{
    Mixed r;
    r.dxy = d1_at(wy, owny, 1, ih);
    __builtin_amdgcn_sched_barrier(0);
    r.dxz = d1_at(wz, ownz, 1, ih);
    __builtin_amdgcn_sched_barrier(0);
    r.dyz = d1_at(wz, ownz, RS, ih);
    return r;
}

// chunks of PAIR_CHUNK consecutive pairs are dealt to the XCDs in turn (workgroup i runs on XCD i mod 8)
__device__ __forceinline__ int64_t pair_of_workgroup(int64_t wg)
{
    const int64_t x = wg % NXCD, q = wg / NXCD;
    return (q / PAIR_CHUNK) * (PAIR_CHUNK * NXCD) + x * PAIR_CHUNK + (q % PAIR_CHUNK);
}

}  // namespace pr

// A block whose x sibling is subdivided has no partner.  It runs here too, as the first half of a brick whose second
// half is a phantom: the first three columns of that half are the block's own ghost points beyond its upper x
// face (taken through the block's own table row), the rest is filled with any valid value, and the threads of the
// second half go through all the motions (they must meet the barriers) but write nothing to memory.
template <int EPI>
__global__ __launch_bounds__(pr::NT) void k_rhs_pair(DeviceTree tr, RhsArgs a)
{
    __shared__ double tile[pr::TILE];
    __shared__ double wyz[pr::WZ + pr::WY];          // D1_z u and D1_y u during the second-derivative passes
    __shared__ double lapS[10 * pr::NT];             // Lap_s of the thread's point at lapS[s * pr::NT + tid]
    __shared__ double keep10[pr::NT];                // u_10 at the thread's point, from pass 0 to the pass over variable 23
    double* const wz = wyz;
    double* const wy = wyz + pr::WZ;
    static_assert(3 * pr::NT <= pr::WZ + pr::WY, "u_23, u_22, u_21 are kept in the idle D1 arrays");
    __shared__ int32_t gt[2 * 27 * 5];               // table rows of the two blocks
    __shared__ uint32_t s_level;

    const int64_t q = pr::pair_of_workgroup(blockIdx.x);
    if (q >= tr.n_units) return;                     // uniform
    const int tid = threadIdx.x;
    const int32_t unit = tr.units[q];
    const bool single = unit & kUnitSingle;          // uniform
    const int64_t b0 = unit & ~kUnitSingle, nb = tr.nb;
    // the rows of b0 and b0 + 1 are adjacent; a single block's row twice
    if (tid < 2 * 27 * 5) gt[tid] = tr.ghost_v[b0 * (27 * 5) + (single && tid >= 27 * 5 ? tid - 27 * 5 : tid)];
    if (tid == 320) s_level = tr.leaves[b0].level;
    __syncthreads();

    // thread -> point: the upper half of the workgroup takes the second block; inside a block lanes run over (i, k)
    // and the wavefront number is j, as in the one-block kernel
    const int half = tid >> 9, t9 = tid & 511;
    const int i = t9 & 7, k = (t9 >> 3) & 7, j = t9 >> 6;
    const int xi = i + NPT * half;                   // 0..15 along the brick
    const int c = (k + PAD) * pr::PS + (j + PAD) * pr::RS + (xi + PAD);
    const bool phantom = single && half;             // uniform over a wavefront
    // byte offset of the thread's point inside one variable's zipped array (phantom: of the same point of the real block,
    // so that everything it loads exists)
    const uint32_t o8 = ((uint32_t)(b0 + (single ? 0 : half)) * BLK + (k * NPT + j) * NPT + i) * 8u;
    const int lvl = __builtin_amdgcn_readfirstlane((int)s_level);
    const double ih = __longlong_as_double((long long)(1026 + lvl) << 52), ih2 = __longlong_as_double((long long)(1029 + 2 * lvl) << 52);
    const double sigma = a.sigma;

    // fill plan, in registers: source offset (bit 0: virtual block) and tile index of the thread's ghost points, and the
    // source of its own point
    uint32_t gsrc[pr::USE_EDGE];
    int gdst[pr::USE_EDGE];
    auto source = [&](int ii, int jj, int kk) -> uint32_t {
        int h = ii >= PAD + NPT ? 1 : 0;             // which block's table row: its own part of x and the ghosts beyond it
        int rx = h ? (ii < PAD + 2 * NPT ? 1 : 2) : (ii < PAD ? 0 : 1);
        const int ry = jj < PAD ? 0 : (jj < PAD + NPT ? 1 : 2);
        const int rz = kk < PAD ? 0 : (kk < PAD + NPT ? 1 : 2);
        int lx = ii - PAD - NPT * h + (1 - rx) * NPT;
        const int ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
        if (single && h) {
            if (ii >= 2 * PAD + NPT) return (uint32_t)b0 * (BLK * 8u);   // phantom region: the real block's first value
            h = 0; rx = 2; lx = ii - PAD - NPT;      // the real block's ghost columns beyond its upper x face
        }
        return ghost_source(&gt[h * (27 * 5) + (rz * 9 + ry * 3 + rx) * 5], rx, ry, rz, lx, ly, lz);
    };
#pragma unroll
    for (int m = 0; m < pr::USE_EDGE; ++m) {
        int ii, jj, kk;
        pr::ghost_point(tid + m * pr::NT, ii, jj, kk);
        gsrc[m] = source(ii, jj, kk);
        gdst[m] = kk * pr::PS + jj * pr::RS + ii;
    }
    const uint32_t own_src = phantom ? source(xi + PAD, j + PAD, k + PAD) : o8;
    // in a pass that reads the faces only, the second entry of the threads past the face prefix is masked
    const bool face_mask1 = tid + pr::NT >= pr::NGF;

    auto var_base = [&](int v) -> const double* { return a.in + (int64_t)v * nb * BLK; };
    auto virt_base = [&](int v) -> const double* { return a.virt + (int64_t)v * tr.n_virt * BLK; };
    auto centre = [&](int v) -> double { return ldg(var_base(v), o8); };

    struct Fetch { double own, g[pr::USE_EDGE]; };
    // request variable v's tile data: the thread's own point and its ghost points
    auto prefetch = [&](Fetch& f, int v, auto use) {
        constexpr int USE = decltype(use)::value;
        const double* base = var_base(v);
        const double* vbase = virt_base(v);
        f.own = ldg((own_src & 1u) ? vbase : base, own_src & ~1u);
#pragma unroll
        for (int m = 0; m < USE; ++m) {
            uint32_t off = gsrc[m];
            if (USE == pr::USE_FACE && m == 1 && face_mask1) off = 0;
            f.g[m] = ldg((off & 1u) ? vbase : base, off & ~1u);
        }
    };
    auto commit = [&](const Fetch& f, auto use) {
        constexpr int USE = decltype(use)::value;
        tile[c] = f.own;
#pragma unroll
        for (int m = 0; m < USE; ++m) {
            int d = gdst[m];
            if (USE == pr::USE_FACE && m == 1 && face_mask1) d = pr::DUMMY;
            tile[d] = f.g[m];
        }
    };
    using UseEdge = std::integral_constant<int, pr::USE_EDGE>;
    using UseFace = std::integral_constant<int, pr::USE_FACE>;

    // Point-wise factors.  alpha and beta are kept as the fields' own values u_0..u_3, so that the same registers also
    // serve as the operand u_{a+11} of the passes a = 13..16.  The other passes that need a variable already seen take
    // it from LDS where there is room (u_10 from pass 0; u_23, u_22, u_21 from the passes over them, parked in the D1
    // arrays, which are idle by then); the passes a = 0..9, whose operand comes later in the stream, and a = 17..22
    // (u_4..u_9, which live on only as G) read it from memory.
    const double u0 = centre(0), bx = centre(1), by = centre(2), bz = centre(3);
    const double Gxx = 1.0 - 0.125 * centre(4), Gxy = -(0.125 * centre(5)), Gxz = -(0.125 * centre(6));
    const double Gyy = 1.0 - 0.125 * centre(7), Gyz = -(0.125 * centre(8)), Gzz = 1.0 - 0.125 * centre(9);
    double nx = 0, ny = 0, nz = 0;
    const int ownz = k * pr::PS + (j + PAD) * pr::RS + (xi + PAD), owny = k * pr::YPS + j * pr::RS + (xi + PAD);
    Fetch nxt;

    {   // pass 0: gradient of variable 10 only
        const int f = syn24_stream(0), f1 = syn24_stream(1);
        prefetch(nxt, f, UseFace{});
        commit(nxt, UseFace{});
        __syncthreads();
        prefetch(nxt, f1, UseEdge{});
        keep10[tid] = tile[c];
        nx = d1_at(tile, c, 1, ih); ny = d1_at(tile, c, pr::RS, ih); nz = d1_at(tile, c, pr::PS, ih);
        __syncthreads();                             // everybody is done with the tile
        commit(nxt, UseEdge{});
        __syncthreads();
    }
    // passes over the variables with second derivatives (9..0).  The barrier between filling the ghost positions
    // of D1_y u, D1_z u and taking their taps is also the last moment anybody reads the tile.
    auto pass_d2 = [&](int t, auto next_use) {
        const int f = syn24_stream(t), f1 = syn24_stream(t + 1);
        prefetch(nxt, f1, next_use);
        const double unext = centre((f + 11) % 24);
        const EpiOperands eo = with_u<EPI>(epi_prefetch<EPI, true>(a, nb, f, o8), tile[c]);
        const Syn24Part p = syn24_axes<true, pr::RS, pr::PS>(tile, c, wy, wz, owny, ownz, nx, ny, nz, bx, by, bz, Gxx, Gyy, Gzz, sigma, ih, ih2);
        pr::mixed_fill(tile, wy, wz, tid, ih);
        __syncthreads();
        const Mixed mx = pr::mixed_taps(wy, wz, owny, ownz, ih);
        double off = Gxy * mx.dxy;
        off = fma(Gxz, mx.dxz, off);
        off = fma(Gyz, mx.dyz, off);
        const double lap = fma(2.0, off, p.diag);
        lapS[f * pr::NT + tid] = lap;
        if (!phantom) emit<EPI>(a, nb, f, b0, o8, 0u, syn24_combine(p, f, lap, 0.5 * u0, unext), eo);
        commit(nxt, next_use);
        __syncthreads();                             // the tile is complete; D1_y u, D1_z u may be overwritten
    };
#pragma unroll 1
    for (int t = 1; t < 10; ++t) pass_d2(t, UseEdge{});
    pass_d2(10, UseFace{});
    // passes over the variables without second derivatives (23..10); `unext` = u_{a+11} at the thread's point
    auto pass_light = [&](int t, double unext) {
        const int f = syn24_stream(t);
        const bool more = t + 1 < NSTREAM;
        if (more) prefetch(nxt, syn24_stream(t + 1), UseFace{});
        const EpiOperands eo = with_u<EPI>(epi_prefetch<EPI, true>(a, nb, f, o8), tile[c]);
        if (t <= 13) wyz[(t - 11) * pr::NT + tid] = tile[c];     // u_23, u_22, u_21 for the last three passes
        const Syn24Part p = syn24_axes<false, pr::RS, pr::PS>(tile, c, wy, wz, owny, ownz, nx, ny, nz, bx, by, bz, 0.0, 0.0, 0.0, sigma, ih, ih2);
        if (!phantom) emit<EPI>(a, nb, f, b0, o8, 0u, syn24_combine(p, f, lapS[(f % 10) * pr::NT + tid], 0.5 * u0, unext), eo);
        if (more) {
            __syncthreads();                         // everybody is done with the tile
            commit(nxt, UseFace{});
            __syncthreads();
        }
    };
    // u_{a+11}: a = 23 -> u_10 (LDS); a = 22..17 -> u_9..u_4 (memory); a = 16..13 -> u_3..u_0 (registers);
    // a = 12, 11, 10 -> u_23, u_22, u_21 (LDS)
    pass_light(11, keep10[tid]);
#pragma unroll 1
    for (int t = 12; t <= 17; ++t) pass_light(t, centre(21 - t));
    pass_light(18, bz);
    pass_light(19, by);
    pass_light(20, bx);
    pass_light(21, u0);
#pragma unroll 1
    for (int t = 22; t < NSTREAM; ++t) pass_light(t, wyz[(t - 22) * pr::NT + tid]);
}

}  // namespace

hipError_t launch_rhs_pairs(const DeviceTree& t, Epilogue ep, const RhsArgs& a, hipStream_t s)
{
    if (t.n_units <= 0) return hipSuccess;
    if (!a.virt && t.n_virt > 0) return hipErrorInvalidValue;
    const int64_t span = pr::PAIR_CHUNK * NXCD;
    const dim3 grid((unsigned)((t.n_units + span - 1) / span * span)), block(pr::NT);
    switch (ep) {
    case kOutZipped: hipLaunchKernelGGL(k_rhs_pair<kOutZipped>, grid, block, 0, s, t, a); break;
    case kRkFirst: hipLaunchKernelGGL(k_rhs_pair<kRkFirst>, grid, block, 0, s, t, a); break;
    case kRkMiddle: hipLaunchKernelGGL(k_rhs_pair<kRkMiddle>, grid, block, 0, s, t, a); break;
    case kRkLast: hipLaunchKernelGGL(k_rhs_pair<kRkLast>, grid, block, 0, s, t, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace octfd
