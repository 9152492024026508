// LDS tile of one block and one variable: geometry, per-block table rows, the order in which the
// tile is filled ("fill plan"), global-memory access helpers and the workgroup -> block mapping.
// Private to kernels.hip (internal linkage throughout).
#pragma once
#include "kernels.hpp"
#include "lagrange.hpp"

namespace octfd {
namespace {

constexpr int NPT = 8, PAD = 3, NP = 14, BLK = 512, PBLK = 2744;
constexpr int NTHREADS = 512;
constexpr int K_SAME = 0, K_VIRT = 3;   // kinds of a ghost-table entry that are plain copies (1: finer, injection)

// LDS geometry (in doubles).  Rows are stored compactly (stride 14) and planes are padded to a
// stride of 200 = 8 (mod 32).  A wavefront holds one j row of the block, its lanes run over
// (i, k): the eight x-contiguous values of four consecutive k planes then fall into 32 different
// 8-byte banks, and shifting the access by any stencil offset keeps that property.
// wavefronts per SIMD the right-hand-side kernels are compiled for: the 24-field kernel 4 (128 VGPRs per lane, two
// workgroups share a compute unit, which is also what its LDS allows); the other kinds 8 (64 VGPRs, four workgroups)
constexpr int waves_per_simd(int kind) { return kind == OT_RHS_SYN24 ? 4 : 8; }
constexpr int RS = NP;                   // 14
constexpr int PS = NP * RS + 4;          // 200
constexpr int TILE = NP * PS;            // 14 planes
constexpr int WZ = NPT * PS;             // D1_z u on [8 k][14 jj][14 ii]
constexpr int YPS = NPT * RS + 8;        // plane stride of the D1_y array, 120 = 24 (mod 32)
constexpr int WY = NPT * YPS;            // D1_y u on [8 k][8 j][14 ii]
struct BlockInfo {       // per-workgroup copy of the block's table row
    int32_t gt[27 * 5];  // ghost table in which coarser neighbours appear as virtual blocks
    uint32_t level;
};

__device__ __forceinline__ int tidx(int kk, int jj, int ii) { return kk * PS + jj * RS + ii; }

// thread -> interior point: lanes run over (i, k), the wavefront number is j.
__device__ __forceinline__ void point_of(int tid, int& i, int& j, int& k)
{
    i = tid & 7;
    k = (tid >> 3) & 7;
    j = tid >> 6;
}

// Loads and stores of global arrays use a uniform 64-bit base (one variable's array) plus a 32-bit
// byte offset held per thread, so that no per-access 64-bit address arithmetic is needed.  The
// library refuses trees with 2^20 blocks or more, which keeps every offset below 2^32.
// The empty asm keeps the 32-bit offset a 32-bit register at the point of use; otherwise the
// compiler widens the offsets to 64 bits once, outside the variable loop, which doubles their
// register cost and forces a 64-bit add per access.
__device__ __forceinline__ double ldg(const double* base, uint32_t byte_off)
{
    asm volatile("" : "+v"(byte_off));
    return *reinterpret_cast<const double*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ void stg(double* base, uint32_t byte_off, double v)
{
    asm volatile("" : "+v"(byte_off));
    *reinterpret_cast<double*>(reinterpret_cast<char*>(base) + byte_off) = v;
}

// Workgroups are handed to the eight XCDs (each with its own L2) round-robin by workgroup id.
// Chunks of 16 Morton-consecutive blocks (two sibling octets) are dealt to the XCDs in turn: blocks
// that run at the same time on one XCD are then close neighbours, which read each other's rows
// through the same L2, while every XCD still sees the same mix of cheap and expensive blocks.
// (Measured on the 102,075-block tree: 78.0 ms per step against 83.5 ms with one contiguous eighth
// of the Morton order per XCD and 78.4 ms with no remapping.)
constexpr int NXCD = kSchedXcds, XCD_CHUNK = kSchedChunk;
__device__ __forceinline__ int64_t block_of_workgroup(int64_t wg)
{
    const int64_t x = wg % NXCD, q = wg / NXCD;
    return (q / XCD_CHUNK) * (XCD_CHUNK * NXCD) + x * XCD_CHUNK + (q % XCD_CHUNK);   // may be >= nb: caller checks
}
inline unsigned grid_for_blocks(int64_t nb)
{
    const int64_t span = XCD_CHUNK * NXCD;
    return (unsigned)((nb + span - 1) / span * span);
}

__device__ __forceinline__ void load_block_info(BlockInfo& bi, const DeviceTree& tr, int64_t b, int tid)
{
    if (tid < 27 * 5) bi.gt[tid] = tr.ghost_v[b * (27 * 5) + tid];
    if (tid == 320) bi.level = tr.leaves[b].level;
}

// ---------------------------------------------------------------- fill plan

// The 2,744 points of the tile are enumerated so that a prefix of the enumeration is exactly what a
// kernel needs:
//   [0, NFACE)      interior and the six face slabs: all that stencils along the axes read;
//   [NFACE, NEDGE)  the twelve edge slabs: read in addition by the mixed second derivatives;
//   [NEDGE, PBLK)   the eight corners: needed only when the whole padded block is written out.
// Fetching only the prefix in use matters because every 8-point ghost row is a 64-byte half of a
// 128-byte line of the neighbour's zipped storage, of which an x ghost uses three values: faces
// alone touch 288 rows per tile (152 lines), faces and edges 516 rows (288 lines), the full tile
// 588 rows (336 lines).
constexpr int NFACE = BLK + 6 * PAD * NPT * NPT;                 // 1664
constexpr int NEDGE = NFACE + 12 * PAD * PAD * NPT;              // 2528
constexpr int PLAN_FACE = (NFACE + NTHREADS - 1) / NTHREADS;     // 4 entries per thread
constexpr int PLAN_EDGE = (NEDGE + NTHREADS - 1) / NTHREADS;     // 5
constexpr int PLAN_FULL = (PBLK + NTHREADS - 1) / NTHREADS;      // 6

__device__ __forceinline__ int ghost_index(int g) { return g < PAD ? g : g + NPT; }   // 0,1,2,11,12,13

__device__ __forceinline__ void tile_point(int p, int& ii, int& jj, int& kk)
{
    if (p < 14 * 64) {                               // x-extended interior rows
        const int r = p / NP;
        ii = p - r * NP; jj = PAD + (r & 7); kk = PAD + (r >> 3);
    } else if (p < 14 * 64 + 384) {                  // y faces
        const int q = p - 14 * 64, r = q >> 3, kq = r / 6;
        ii = PAD + (q & 7); jj = ghost_index(r - 6 * kq); kk = PAD + kq;
    } else if (p < NFACE) {                          // z faces
        const int q = p - (14 * 64 + 384);
        ii = PAD + (q & 7); jj = PAD + ((q >> 3) & 7); kk = ghost_index(q >> 6);
    } else if (p < NFACE + 288) {                    // xy edges
        const int q = p - NFACE, r = q / 6, kq = r / 6;
        ii = ghost_index(q - 6 * r); jj = ghost_index(r - 6 * kq); kk = PAD + kq;
    } else if (p < NFACE + 576) {                    // xz edges
        const int q = p - (NFACE + 288), r = q / 6;
        ii = ghost_index(q - 6 * r); jj = PAD + (r & 7); kk = ghost_index(r >> 3);
    } else if (p < NEDGE) {                          // yz edges
        const int q = p - (NFACE + 576), r = q >> 3, kq = r / 6;
        ii = PAD + (q & 7); jj = ghost_index(r - 6 * kq); kk = ghost_index(kq);
    } else {                                         // corners
        const int q = p - NEDGE, r = q / 6, kq = r / 6;
        ii = ghost_index(q - 6 * r); jj = ghost_index(r - 6 * kq); kk = ghost_index(kq);
    }
}

// Entries with nothing to copy (beyond the range in use, or interpolated later) read element 0 and
// write to DUMMY, a padding slot of the tile that no stencil reads; the copy loop is branch-free.
constexpr int DUMMY = NP * RS;   // first padding slot behind plane 0
// src: byte offset in the source array.  It is needed once per variable: the 24-field kernel, short of
// registers, keeps it in LDS as src[m * NTHREADS + tid]; with REG the entries are registers (the other
// kinds: 8 KB less LDS, which lets a fourth workgroup onto the compute unit).
// dst: tile index, two 16-bit values per register.
template <int NPLAN, bool REG = false>
struct FillPlan {
    uint32_t* src;
    uint32_t srcr[REG ? NPLAN : 1];
    uint32_t dstp[(NPLAN + 1) / 2];
    __device__ __forceinline__ uint32_t get_src(int m, int tid) const { return REG ? srcr[m] : src[m * NTHREADS + tid]; }
    __device__ __forceinline__ void set_src(int m, int tid, uint32_t v) { if (REG) srcr[m] = v; else src[m * NTHREADS + tid] = v; }
    __device__ __forceinline__ int dst(int m) const { return (dstp[m >> 1] >> (16 * (m & 1))) & 0xffff; }
    __device__ __forceinline__ void set_dst(int m, int v) { dstp[m >> 1] = (m & 1) ? (dstp[m >> 1] | ((uint32_t)v << 16)) : (uint32_t)v; }
};
static_assert(TILE < 65536, "tile indices are packed in pairs");

// Where the point (lx, ly, lz) of the same-level octant in direction (rx, ry, rz) - 1 comes from, given that
// direction's entry e of the table in which coarser neighbours appear as virtual blocks: byte offset into one variable's zipped array (same level: copy;
// finer: the coinciding node of the child that holds it) or, marked by bit 0, into its array of virtual blocks.
__device__ __forceinline__ uint32_t ghost_source(const int32_t* e, int rx, int ry, int rz, int lx, int ly, int lz)
{
    const int kind = e[0];
    uint32_t elem;
    if (kind == K_SAME || kind == K_VIRT) {
        elem = (uint32_t)e[1] * BLK + (lz * NPT + ly) * NPT + lx;
    } else {
        // which child holds the point: forced by the direction on non-free axes
        const int bx = rx == 1 ? (lx >> 2) : (rx == 0 ? 1 : 0);
        const int by = ry == 1 ? (ly >> 2) : (ry == 0 ? 1 : 0);
        const int bz = rz == 1 ? (lz >> 2) : (rz == 0 ? 1 : 0);
        int q = 0, sh = 0;
        if (rx == 1) { q |= bx << sh; ++sh; }
        if (ry == 1) { q |= by << sh; ++sh; }
        if (rz == 1) { q |= bz << sh; }
        elem = (uint32_t)e[1 + q] * BLK + ((2 * lz - NPT * bz) * NPT + (2 * ly - NPT * by)) * NPT + (2 * lx - NPT * bx);
    }
    return elem * 8u | (kind == K_VIRT ? 1u : 0u);
}

// Source of every padded point this thread fills, as a byte offset into one variable's zipped
// array (same-level copy or injection from a finer leaf) or, for a point inside a virtual block, into
// one variable's part of the array of virtual blocks, marked by bit 0 (offsets are multiples of 8).
// NPOINTS = how long a prefix of the enumeration is planned.
template <int NPLAN, int NPOINTS, bool REG>
__device__ __forceinline__ void make_plan_zipped(FillPlan<NPLAN, REG>& fp, const BlockInfo& bi, int tid)
{
#pragma unroll
    for (int m = 0; m < NPLAN; ++m) {
        const int p = tid + m * NTHREADS;
        uint32_t src = 0;
        int dst = DUMMY;
        if (p < NPOINTS) {
            int ii, jj, kk;
            tile_point(p, ii, jj, kk);
            const int rx = ii < PAD ? 0 : (ii < PAD + NPT ? 1 : 2);
            const int ry = jj < PAD ? 0 : (jj < PAD + NPT ? 1 : 2);
            const int rz = kk < PAD ? 0 : (kk < PAD + NPT ? 1 : 2);
            // coordinates inside the neighbouring octant of the same level, 0..7
            const int lx = ii - PAD + (1 - rx) * NPT, ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
            dst = tidx(kk, jj, ii);
            src = ghost_source(&bi.gt[(rz * 9 + ry * 3 + rx) * 5], rx, ry, rz, lx, ly, lz);
        }
        fp.set_src(m, tid, src);
        fp.set_dst(m, dst);
    }
}

// same for a padded source block (plain copy)
template <int NPLAN, int NPOINTS, bool REG>
__device__ __forceinline__ void make_plan_padded(FillPlan<NPLAN, REG>& fp, int tid)
{
#pragma unroll
    for (int m = 0; m < NPLAN; ++m) {
        const int p = tid + m * NTHREADS;
        const bool ok = p < NPOINTS;
        int ii, jj, kk;
        tile_point(ok ? p : 0, ii, jj, kk);
        fp.set_src(m, tid, ok ? (uint32_t)((kk * NP + jj) * NP + ii) * 8u : 0u);
        fp.set_dst(m, ok ? tidx(kk, jj, ii) : DUMMY);
    }
}

}  // namespace
}  // namespace octfd
