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
#include "lagrange.hpp"

#include <type_traits>

namespace octfd {
namespace {

constexpr int NPT = 8, PAD = 3, NP = 14, BLK = 512, PBLK = 2744;
constexpr int NTHREADS = 512;
constexpr int K_COARSER = 2, K_SAME = 0;

// LDS geometry (in doubles).  Rows are stored compactly (stride 14) and planes are padded to a
// stride of 200 = 8 (mod 32).  A wavefront holds one j row of the block, its lanes run over
// (i, k): the eight x-contiguous values of four consecutive k planes then fall into 32 different
// 8-byte banks, and shifting the access by any stencil offset keeps that property.
constexpr int WAVES_PER_SIMD = 4;        // 128 VGPRs per lane: two workgroups of the stage kernels share a compute unit
constexpr int RS = NP;                   // 14
constexpr int PS = NP * RS + 4;          // 200
constexpr int TILE = NP * PS;            // 14 planes
constexpr int WZ = NPT * PS;             // D1_z u on [8 k][14 jj][14 ii]
constexpr int YPS = NPT * RS + 8;        // plane stride of the D1_y array, 120 = 24 (mod 32)
constexpr int WY = NPT * YPS;            // D1_y u on [8 k][8 j][14 ii]
// wy and wz together need 2,560 doubles; the ghost interpolation stages several coarser leaves at
// once in the same area and profits from the 448 more that still let two workgroups share a CU
constexpr int SCRATCH = WZ + WY + 448;

constexpr int ROUND_SRC = 4;                 // source leaves per round (one register each while in flight)
struct BoxPlan {
    int32_t nround;
    int32_t rbeg[9];                         // round r covers sources rbeg[r] .. rbeg[r+1]-1
    int32_t n1[8], n2[8], n3[8], bstart[8];  // per round: items of the x / y / z pass, start of region B
    int32_t o1[8], o2[8], o3[8];             // per source: offset of its items inside its round's pass
    uint32_t mx[8], mpl[8];                  // per source: magic numbers for dividing by nx and by nx*ny
    int16_t sx[8], nx[8], sy[8], ny[8], sz[8], nz[8], fx0[8], fy0[8], fz0[8];
    int16_t face_src[6];                     // for the q-th coarser face: which source (index into the list) it is
};

struct BlockInfo {       // per-workgroup copy of the block's table rows
    int32_t gt[27 * 5];
    int32_t cs[32];      // [0..15] coarse sources: {leaf id, packed region range} x 8, id < 0 ends the
                         // list; [16] number of coarser faces, [17..28] {face, leaf id} pairs
    int32_t slot[8];     // centred ghost rule: where the padded block of coarse source s sits (src_slot of its id)
    uint32_t level, ax, ay, az;
    double lag[36];
    BoxPlan box;         // filled by make_box_plan()
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
constexpr int NXCD = 8, XCD_CHUNK = 16;
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
    if (tid < 27 * 5) bi.gt[tid] = tr.ghost[b * (27 * 5) + tid];
    if (tid >= 192 && tid < 192 + 36) bi.lag[tid - 192] = c_lag[tid - 192];
    if (tid >= 256 && tid < 256 + 32) bi.cs[tid - 256] = tr.coarse[b * 32 + (tid - 256)];
    if (tid >= 384 && tid < 384 + 8) {
        const int32_t id = tr.coarse[b * 32 + 2 * (tid - 384)];
        bi.slot[tid - 384] = id >= 0 ? tr.src_slot[id] : -1;
    }
    if (tid == 320) {
        const ot_leaf lf = tr.leaves[b];
        bi.level = lf.level; bi.ax = lf.ix; bi.ay = lf.iy; bi.az = lf.iz;
    }
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
// src: byte offset in the source array, kept in LDS as src[m * NTHREADS + tid] (it is needed once
// per variable and registers are scarce); dst: tile index, two 16-bit values per register
template <int NPLAN>
struct FillPlan {
    uint32_t* src;
    uint32_t dstp[(NPLAN + 1) / 2];
    __device__ __forceinline__ int dst(int m) const { return (dstp[m >> 1] >> (16 * (m & 1))) & 0xffff; }
    __device__ __forceinline__ void set_dst(int m, int v) { dstp[m >> 1] = (m & 1) ? (dstp[m >> 1] | ((uint32_t)v << 16)) : (uint32_t)v; }
};
static_assert(TILE < 65536, "tile indices are packed in pairs");
static_assert(SCRATCH >= 1024 + 2 * 512, "face interpolation staging: 8 x 128 per-wavefront + 2 x 512 shared");

// Source of every padded point this thread fills, as a byte offset into one variable's zipped
// array (same-level copy or injection from a finer leaf).  Points whose source is coarser are left
// to the interpolation passes.  NPOINTS = how long a prefix of the enumeration is planned.
template <int NPLAN, int NPOINTS>
__device__ __forceinline__ void make_plan_zipped(FillPlan<NPLAN>& fp, const BlockInfo& bi, int tid)
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
            const int32_t* e = &bi.gt[(rz * 9 + ry * 3 + rx) * 5];
            const int kind = e[0];
            if (kind != K_COARSER) {
                // coordinates inside the neighbouring octant of the same level, 0..7
                const int lx = ii - PAD + (1 - rx) * NPT, ly = jj - PAD + (1 - ry) * NPT, lz = kk - PAD + (1 - rz) * NPT;
                dst = tidx(kk, jj, ii);
                uint32_t elem;
                if (kind == K_SAME) {
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
                src = elem * 8u;
            }
        }
        fp.src[m * NTHREADS + tid] = src;
        fp.set_dst(m, dst);
    }
}

// same for a padded source block (plain copy)
template <int NPLAN, int NPOINTS>
__device__ __forceinline__ void make_plan_padded(FillPlan<NPLAN>& fp, int tid)
{
#pragma unroll
    for (int m = 0; m < NPLAN; ++m) {
        const int p = tid + m * NTHREADS;
        const bool ok = p < NPOINTS;
        int ii, jj, kk;
        tile_point(ok ? p : 0, ii, jj, kk);
        fp.src[m * NTHREADS + tid] = ok ? (uint32_t)((kk * NP + jj) * NP + ii) * 8u : 0u;
        fp.set_dst(m, ok ? tidx(kk, jj, ii) : DUMMY);
    }
}


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
// done by one thread per block, once: boxes from the packed region ranges, greedy rounds in list order
__device__ void make_box_plan(BlockInfo& bi)
{
    BoxPlan& bp = bi.box;
    int nr = 0, sumc = 0, sum1 = 0, sum2 = 0, sum3 = 0, ns = 0;
    bp.rbeg[0] = 0;
    for (int s = 0; s < 8; ++s) {
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

// every coarser source leaf of the block, one after the other; pbase = one variable's compact array of
// padded source leaves (or, with by_id, the padded array of all blocks)
template <bool BY_ID = false>
__device__ __forceinline__ void interp_boxes_centred(double* tile, double* scratch, const BlockInfo& bi,
                                                     const double* __restrict__ pbase, int tid)
{
    const BoxPlan& bp = bi.box;
    const int ns = bp.rbeg[bp.nround];
    auto box = [&](CentredBox& cb, int s) {
        const int64_t src = BY_ID ? bi.cs[2 * s] : bi.slot[s];
        cb.set(bi, pbase + src * PBLK, bp.sx[s], bp.nx[s], bp.sy[s], bp.ny[s], bp.sz[s], bp.nz[s]);
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
// the same where only the face slabs of the tile are read: one 3 x 8 x 8 box per coarser face
__device__ __forceinline__ void interp_faces_centred(double* tile, double* scratch, const BlockInfo& bi,
                                                     const double* __restrict__ pbase, int tid)
{
    const int n = bi.cs[16];
    auto box = [&](CentredBox& cb, int q) {
        const int face = bi.cs[17 + 2 * q], ax = face >> 1, s0 = (face & 1) ? PAD + NPT : 0;
        cb.set(bi, pbase + (int64_t)bi.slot[bi.box.face_src[q]] * PBLK, ax == 0 ? s0 : PAD, ax == 0 ? PAD : NPT,
               ax == 1 ? s0 : PAD, ax == 1 ? PAD : NPT, ax == 2 ? s0 : PAD, ax == 2 ? PAD : NPT);
    };
    if (n == 0) return;
    CentredBox cur, nxt;
    double c[2];
    box(cur, 0);
    cur.request(c, tid);
#pragma unroll 1
    for (int q = 0; q < n; ++q) {
        cur.stage(scratch, c, tid);
        if (q + 1 < n) { box(nxt, q + 1); nxt.request(c, tid); }
        cur.sweep(tile, scratch, bi, tid);
        cur = nxt;
    }
}

// Filling the tile of one variable is split in two so that the global loads of the next variable
// can be in flight while the current one is being differentiated:
//   prefetch(): issue the planned loads into registers;
//   commit():   store them into a tile buffer, then (zipped input only) interpolate what comes from
//               coarser leaves.  `base` is that variable's zipped array (ZIN) or this block's padded
//               data.  All threads call both.  commit() does NOT end with a barrier.
// USE = how many plan entries per thread are in use (PLAN_FACE: faces only).
template <int NPLAN, int USE>
__device__ __forceinline__ void prefetch(double (&v)[NPLAN], const FillPlan<NPLAN>& fp, const double* __restrict__ base, int tid)
{
    uint32_t off[USE];
#pragma unroll
    for (int m = 0; m < USE; ++m) off[m] = fp.src[m * NTHREADS + tid];
    // the last entry in use may reach beyond the face prefix: read element 0 instead
    if (USE == PLAN_FACE && NPLAN > PLAN_FACE && tid + (USE - 1) * NTHREADS >= NFACE) off[USE - 1] = 0;
#pragma unroll
    for (int m = 0; m < USE; ++m) v[m] = ldg(base, off[m]);
}

// Values of the coarser face neighbours can be requested together with the tile data
// (coarse_prefetch) so that their latency hides behind the stencil work: CPRE slots, in the order of
// the block's coarse-face list; further faces are loaded late.
constexpr int CPRE = 3;
__device__ __forceinline__ void coarse_prefetch(double (&cv)[CPRE], const BlockInfo& bi, const double* __restrict__ base, int tid)
{
    const int n = bi.cs[16];
#pragma unroll
    for (int q = 0; q < CPRE; ++q)
        if (q < n) cv[q] = ldg(base, ((uint32_t)bi.cs[18 + 2 * q] * BLK + tid) * 8u);
}

// CENTRED: ghost values from coarser leaves follow the centred rule and come from pbase (that
// variable's padded source leaves).
template <bool ZIN, int NPLAN, int USE, bool CENTRED = false>
__device__ __forceinline__ void commit(double* tile, double* scratch, const BlockInfo& bi, const FillPlan<NPLAN>& fp,
                                       const double (&v)[NPLAN], const double (&cv)[CPRE], bool have_cv,
                                       const double* __restrict__ base, int tid, const double* __restrict__ pbase = nullptr)
{
#pragma unroll
    for (int m = 0; m < USE; ++m) {
        int d = fp.dst(m);
        if (USE == PLAN_FACE && NPLAN > PLAN_FACE && m == USE - 1 && tid + m * NTHREADS >= NFACE) d = DUMMY;
        tile[d] = v[m];
    }
    if (!ZIN || bi.cs[0] < 0) return;
    // Control flow below is uniform over the workgroup.
    if (CENTRED) {
        if (USE == PLAN_FACE) interp_faces_centred(tile, scratch, bi, pbase, tid);
        else interp_boxes_centred(tile, scratch, bi, pbase, tid);
    } else if (USE == PLAN_FACE) {
        // Faces only: each face neighbour that is coarser supplies a 3 x 8 x 8 slab.  Wavefront w
        // owns the coarse plane cz = w: it interpolates that plane in x and then in y out of its
        // own staging area with no workgroup barrier; only the z pass, which combines the planes,
        // needs one.  The y-pass results are double-buffered across faces.
        const int n = bi.cs[16];
        const int wave = tid >> 6, lane = tid & 63;
        double* Cs = scratch + wave * 128;       // this wavefront's coarse plane, [cy][cx]
        double* T1s = Cs + 64;                   // after the x pass, [cy][tx]
        __syncthreads();                         // the staging arrays may still be read as wy / wz
#pragma unroll 1
        for (int q = 0; q < n; ++q) {
            const int face = bi.cs[17 + 2 * q], ax = face >> 1, s0 = (face & 1) ? PAD + NPT : 0;
            const int sx = ax == 0 ? s0 : PAD, sy = ax == 1 ? s0 : PAD, sz = ax == 2 ? s0 : PAD;
            const int nx = ax == 0 ? PAD : NPT, ny = ax == 1 ? PAD : NPT, nz = ax == 2 ? PAD : NPT;
            const uint32_t mx = div_magic(nx), mxy = div_magic(nx * ny);
            const int fx0 = (NPT * bi.ax + sx + 16 - PAD) & 15;
            const int fy0 = (NPT * bi.ay + sy + 16 - PAD) & 15;
            const int fz0 = (NPT * bi.az + sz + 16 - PAD) & 15;
            double* T2 = scratch + 1024 + (q & 1) * 512;   // after the y pass, [cz][ty][tx], 64 per plane
            double cval;
            if (have_cv && q < CPRE) cval = q == 0 ? cv[0] : (q == 1 ? cv[1] : cv[2]);
            else cval = ldg(base, ((uint32_t)bi.cs[18 + 2 * q] * BLK + tid) * 8u);
            Cs[lane] = cval;
            __builtin_amdgcn_wave_barrier();
            if (lane < NPT * nx) {                                   // x pass, item (cy, tx)
                const int cy = div_by(lane, mx), tx = lane - cy * nx;
                T1s[cy * NPT + tx] = interp_line(&Cs[cy * NPT], 1, fx0 + tx, bi.lag);
            }
            __builtin_amdgcn_wave_barrier();
            if (lane < ny * nx) {                                    // y pass, item (ty, tx)
                const int ty = div_by(lane, mx), tx = lane - ty * nx;
                T2[wave * 64 + lane] = interp_line(&T1s[tx], NPT, fy0 + ty, bi.lag);
            }
            __syncthreads();
            if (tid < nz * ny * nx) {                                // z pass, into the tile
                const int tz = div_by(tid, mxy), r = tid - tz * nx * ny, ty = div_by(r, mx), tx = r - ty * nx;
                tile[tidx(sz + tz, sy + ty, sx + tx)] = interp_line(&T2[r], 64, fz0 + tz, bi.lag);
            }
        }
    } else {
        interp_boxes(tile, scratch, bi, base, tid);
    }
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
    r.ko = sigma * ((kxy + z.ko) * (ih * 0.015625));
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

template <int EPI>
__device__ __forceinline__ EpiOperands epi_prefetch(const RhsArgs& a, int64_t nb, int w, uint32_t o8)
{
    EpiOperands e{0.0, 0.0};
    const int64_t f = (int64_t)w * nb * BLK;
    if (EPI == kRkFirst || EPI == kRkMiddle || EPI == kRkLast) e.u = ldg(a.u + f, o8);
    if (EPI == kRkMiddle || EPI == kRkLast) e.acc = ldg(a.acc + f, o8);
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

// ---------------------------------------------------------------- right-hand-side kernel

// One SYN24 variable at this thread's point, fused axis by axis so that few values are live at any
// time (the scheduling fences keep the compiler from fetching every tap up front).  (nx, ny, nz)
// holds the gradient of the successor variable on entry and this variable's own gradient on exit.
//   t1 = beta . grad u,  t3q = grad u . grad u_next (before the factor 1/4),  ko = dissipation,
//   diag = Gxx Dxx + Gyy Dyy + Gzz Dzz (WITH_D2 only).
// WITH_D2 also publishes D1_y u and D1_z u of the own point for mixed_derivs().
struct Syn24Part { double t1, t3q, ko, diag; };

template <bool WITH_D2>
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
    const AxisOps y = axis_ops<WITH_D2>(t, c, RS, u0, ih, ih2);
    r.t1 = fma(by, y.d1, r.t1);
    r.t3q = fma(y.d1, ny, r.t3q);
    ny = y.d1;
    if (WITH_D2) { r.diag = fma(Gyy, y.d2, r.diag); wy[owny] = y.d1; }
    ksum = ksum + y.ko;
    __builtin_amdgcn_sched_barrier(0);
    const AxisOps z = axis_ops<WITH_D2>(t, c, PS, u0, ih, ih2);
    r.t1 = fma(bz, z.d1, r.t1);
    r.t3q = fma(z.d1, nz, r.t3q);
    nz = z.d1;
    if (WITH_D2) { r.diag = fma(Gzz, z.d2, r.diag); wz[ownz] = z.d1; }
    r.ko = sigma * ((ksum + z.ko) * (ih * 0.015625));
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

template <int KIND, bool ZIN, int EPI, bool CENTRED = false>
__global__ __launch_bounds__(NTHREADS, WAVES_PER_SIMD) void k_rhs(DeviceTree tr, RhsArgs a)
{
    static_assert(ZIN || !CENTRED, "the centred ghost rule applies to zipped input");
    constexpr int NBUF = KIND == OT_RHS_SYN24 ? 2 : 1;
    __shared__ double tiles[NBUF * TILE];
    // SYN24 keeps wy / wz here and stages whole boxes of coarser leaves; the other kinds read face slabs
    // only, whose interpolation needs 2,048 doubles (and lets three workgroups share a compute unit)
    constexpr int FACE_STAGING = 1024 + 2 * 512;
    static_assert(FACE_STAGING >= 810, "centred interpolation of one 3 x 8 x 8 face slab");
    __shared__ double scratch[KIND == OT_RHS_SYN24 ? SCRATCH : (ZIN ? FACE_STAGING : 1)];
    __shared__ BlockInfo bi;
    // second derivatives (SYN24 only) read the edge slabs of the tile too
    constexpr int NPLAN = KIND == OT_RHS_SYN24 ? PLAN_EDGE : PLAN_FACE;
    constexpr int NPOINTS = KIND == OT_RHS_SYN24 ? NEDGE : NFACE;
    __shared__ uint32_t plan_src[NPLAN * NTHREADS];

    const int tid = threadIdx.x;
    const int64_t nb = tr.nb;
    const int64_t b = block_of_workgroup(blockIdx.x);
    if (b >= nb) return;                             // uniform over the workgroup
    load_block_info(bi, tr, b, tid);
    __syncthreads();
    if (tid == 0 && (KIND == OT_RHS_SYN24 || CENTRED)) make_box_plan(bi);   // read only after the next barrier

    int i, j, k;
    point_of(tid, i, j, k);
    const int c = tidx(k + PAD, j + PAD, i + PAD);
    // byte offsets of this thread's point inside one variable's zipped array / inside a padded block
    const uint32_t o8 = ((uint32_t)b * BLK + (k * NPT + j) * NPT + i) * 8u;
    const uint32_t p8 = (((k + PAD) * NP + (j + PAD)) * NP + (i + PAD)) * 8u;
    const double ih = (double)(NPT << bi.level), ih2 = ih * ih;
    const double sigma = a.sigma;

    FillPlan<NPLAN> fp;
    fp.src = plan_src;
    if (ZIN) make_plan_zipped<NPLAN, NPOINTS>(fp, bi, tid);
    else make_plan_padded<NPLAN, NPOINTS>(fp, tid);
    double pv[NPLAN];
    double cv[CPRE];   // values of coarser face neighbours requested ahead (SYN24 first-derivative passes)

    auto var_base = [&](int v) -> const double* {
        return ZIN ? a.in + (int64_t)v * nb * BLK : a.in + ((int64_t)v * nb + b) * PBLK;
    };
    auto pad_base = [&](int v) -> const double* {   // centred rule: variable v's padded source leaves
        return CENTRED ? a.pad_src + (int64_t)v * tr.n_src * PBLK : nullptr;
    };
    auto stage = [&](int v) {   // bring variable v into tile buffer 0 (barrier before and after)
        __syncthreads();
        prefetch<NPLAN, PLAN_FACE>(pv, fp, var_base(v), tid);
        commit<ZIN, NPLAN, PLAN_FACE, CENTRED>(tiles, scratch, bi, fp, pv, cv, false, var_base(v), tid, pad_base(v));
        __syncthreads();
    };
    auto centre = [&](int v) -> double {   // this thread's own value of variable v
        return ZIN ? ldg(a.in + (int64_t)v * nb * BLK, o8) : ldg(a.in + ((int64_t)v * nb + b) * PBLK, p8);
    };

    if (KIND == OT_RHS_DERIVS) {
        stage(0);
        const EpiOperands e0 = epi_prefetch<EPI>(a, nb, 0, o8), e1 = epi_prefetch<EPI>(a, nb, 1, o8);
        const EpiOperands e2 = epi_prefetch<EPI>(a, nb, 2, o8), e3 = epi_prefetch<EPI>(a, nb, 3, o8);
        const PointOps p = point_ops<true>(tiles, c, 0.0, ih, ih2);
        emit<EPI>(a, nb, 0, b, o8, p8, p.dx, e0);
        emit<EPI>(a, nb, 1, b, o8, p8, p.dy, e1);
        emit<EPI>(a, nb, 2, b, o8, p8, p.dz, e2);
        emit<EPI>(a, nb, 3, b, o8, p8, p.lap, e3);
    } else if (KIND == OT_RHS_WAVE) {
        const EpiOperands e0 = epi_prefetch<EPI>(a, nb, 0, o8), e1 = epi_prefetch<EPI>(a, nb, 1, o8);
        stage(0);
        const PointOps pu = point_ops<true>(tiles, c, sigma, ih, ih2);
        stage(1);
        const PointOps pp = point_ops<false>(tiles, c, sigma, ih, ih2);
        emit<EPI>(a, nb, 0, b, o8, p8, pp.u0 + pu.ko, e0);
        emit<EPI>(a, nb, 1, b, o8, p8, pu.lap + pp.ko, e1);
    } else if (KIND == OT_RHS_BURGERS) {
        stage(0);
        const EpiOperands e0 = epi_prefetch<EPI>(a, nb, 0, o8);
        const PointOps p = point_ops<false>(tiles, c, sigma, ih, ih2);
        const double flux = p.u0 * p.dx;
        emit<EPI>(a, nb, 0, b, o8, p8, p.ko - flux, e0);
    } else {
        // SYN24.  The variables are streamed in descending cyclic order (see syn24_stream).  The
        // first ten real passes (variables 9..0) evaluate the second-derivative combinations Lap_s;
        // each thread parks them at its own point in variables 10+s of the `stash` array, from where
        // the later passes (variables 23..10, which need Lap_{a mod 10}) read them back before those
        // slots receive their final values.  Per-thread state thus shrinks to one gradient.
        //
        // The tile is double-buffered and global memory is requested ahead of its use: tile data
        // of the next variable is loaded into registers at the top of a pass and committed to the
        // other LDS buffer at its end (one barrier per pass, plus the one inside mixed_derivs); the
        // pointwise operands of the next pass (RK accumulator and state, u_{a+11}, Lap) likewise.
        double* wz = scratch;
        double* wy = scratch + WZ;
        const double halpha = 0.5 * centre(0), bx = centre(1), by = centre(2), bz = centre(3);
        const double Gxx = 1.0 - 0.125 * centre(4), Gxy = -(0.125 * centre(5)), Gxz = -(0.125 * centre(6));
        const double Gyy = 1.0 - 0.125 * centre(7), Gyz = -(0.125 * centre(8)), Gzz = 1.0 - 0.125 * centre(9);
        double nx = 0, ny = 0, nz = 0;
        const int ownz = k * PS + (j + PAD) * RS + (i + PAD), owny = k * YPS + j * RS + (i + PAD);
        struct Look { double unext, lap; EpiOperands eo; };

        auto stash_base = [&](int v) -> double* {   // where Lap_{v-10} is parked (v = 10..19)
            return EPI == kOutPadded ? a.stash + ((int64_t)v * nb + b) * PBLK : a.stash + (int64_t)v * nb * BLK;
        };
        const uint32_t s8 = EPI == kOutPadded ? p8 : o8;

        // top of pass t: request the tile data of pass t+1 and this pass's own pointwise operands.
        // NEXT_USE says how much of the tile pass t+1 reads (edges only if it takes second derivatives).
        auto issue = [&](int t, int f, Look& l, int& f1, auto next_use) {
            constexpr int NEXT_USE = decltype(next_use)::value;
            if (t + 1 < NSTREAM) {
                f1 = syn24_stream(t + 1);
                prefetch<NPLAN, NEXT_USE>(pv, fp, var_base(f1), tid);
                if (ZIN && !CENTRED && NEXT_USE == PLAN_FACE) coarse_prefetch(cv, bi, var_base(f1), tid);
            }
            l.unext = centre((f + 11) % 24);
            l.eo = epi_prefetch<EPI>(a, nb, f, o8);
            if (t > 10) l.lap = ldg(stash_base(10 + f % 10), s8);
        };
        using UseEdge = std::integral_constant<int, PLAN_EDGE>;
        using UseFace = std::integral_constant<int, PLAN_FACE>;
        // pass over a variable with second derivatives (9..0)
        auto pass_d2 = [&](int t, auto next_use) {
            constexpr int NEXT_USE = decltype(next_use)::value;
            const double* T = tiles + (t & 1) * TILE;
            const int f = syn24_stream(t);
            int f1 = 0;
            Look l{0.0, 0.0, {0.0, 0.0}};
            issue(t, f, l, f1, next_use);
            const Syn24Part p = syn24_axes<true>(T, c, wy, wz, owny, ownz, nx, ny, nz, bx, by, bz, Gxx, Gyy, Gzz, sigma, ih, ih2);
            const Mixed mx = mixed_derivs(T, wy, wz, tid, owny, ownz, ih);
            double off = Gxy * mx.dxy;
            off = fma(Gxz, mx.dxz, off);
            off = fma(Gyz, mx.dyz, off);
            const double lap = fma(2.0, off, p.diag);
            stg(stash_base(10 + f), s8, lap);
            emit<EPI>(a, nb, f, b, o8, p8, syn24_combine(p, f, lap, halpha, l.unext), l.eo);
            commit<ZIN, NPLAN, NEXT_USE, CENTRED>(tiles + ((t + 1) & 1) * TILE, scratch, bi, fp, pv, cv, NEXT_USE == PLAN_FACE, var_base(f1), tid, pad_base(f1));
            __syncthreads();
        };
        // pass over a variable without second derivatives (23..10)
        auto pass_light = [&](int t) {
            const double* T = tiles + (t & 1) * TILE;
            const int f = syn24_stream(t);
            int f1 = 0;
            Look l{0.0, 0.0, {0.0, 0.0}};
            issue(t, f, l, f1, UseFace{});
            const Syn24Part p = syn24_axes<false>(T, c, wy, wz, owny, ownz, nx, ny, nz, bx, by, bz, 0.0, 0.0, 0.0, sigma, ih, ih2);
            emit<EPI>(a, nb, f, b, o8, p8, syn24_combine(p, f, l.lap, halpha, l.unext), l.eo);
            if (t + 1 < NSTREAM) {
                commit<ZIN, NPLAN, PLAN_FACE, CENTRED>(tiles + ((t + 1) & 1) * TILE, scratch, bi, fp, pv, cv, true, var_base(f1), tid, pad_base(f1));
                __syncthreads();
            }
        };

        {   // pass 0: gradient of variable 10 only
            const int f = syn24_stream(0), f1 = syn24_stream(1);
            prefetch<NPLAN, PLAN_FACE>(pv, fp, var_base(f), tid);
            if (CENTRED) __syncthreads();            // the box plan, made by one thread, is read in this commit already
            commit<ZIN, NPLAN, PLAN_FACE, CENTRED>(tiles, scratch, bi, fp, pv, cv, false, var_base(f), tid, pad_base(f));
            __syncthreads();
            prefetch<NPLAN, PLAN_EDGE>(pv, fp, var_base(f1), tid);
            nx = d1_at(tiles, c, 1, ih); ny = d1_at(tiles, c, RS, ih); nz = d1_at(tiles, c, PS, ih);
            commit<ZIN, NPLAN, PLAN_EDGE, CENTRED>(tiles + TILE, scratch, bi, fp, pv, cv, false, var_base(f1), tid, pad_base(f1));
            __syncthreads();
        }
#pragma unroll 1
        for (int t = 1; t < 10; ++t) pass_d2(t, UseEdge{});
        pass_d2(10, UseFace{});
#pragma unroll 1
        for (int t = 11; t < NSTREAM; ++t) pass_light(t);
    }
}

// ---------------------------------------------------------------- unzip / zip kernels

__global__ __launch_bounds__(NTHREADS) void k_unzip(DeviceTree tr, int nvar, const double* __restrict__ zipped, double* __restrict__ padded)
{
    __shared__ double tile[TILE];
    __shared__ double scratch[SCRATCH];
    __shared__ BlockInfo bi;
    const int tid = threadIdx.x;
    // Workgroup r + G b fills the padded blocks of variables r, r + G, r + 2G, ... of block b, G =
    // min(8, nvar).  With the workgroups dealt to the eight XCDs in turn, an XCD sees a fixed subset of
    // the variables for consecutive blocks one after the other, so a ghost row it fetches was, or soon
    // will be, an interior row of a block it handles for the same variable and is served by its L2
    // (102,075-block tree, 24 variables: 22 GB fetched per call against 77 GB with the blocks of one
    // variable launched together).  The fill plan is built once per workgroup and kept in registers.
    const int stride = nvar < NXCD ? nvar : NXCD;
    const int64_t b = blockIdx.x / stride, nb = tr.nb;
    const int v0 = (int)(blockIdx.x - b * stride);
    load_block_info(bi, tr, b, tid);
    __syncthreads();
    if (tid == 0) make_box_plan(bi);
    FillPlan<PLAN_FULL> fp;
    fp.src = reinterpret_cast<uint32_t*>(scratch);   // the staging area is free until the first interpolation
    make_plan_zipped<PLAN_FULL, PBLK>(fp, bi, tid);
    uint32_t off[PLAN_FULL];
    int from[PLAN_FULL];
#pragma unroll
    for (int m = 0; m < PLAN_FULL; ++m) {
        off[m] = fp.src[m * NTHREADS + tid];             // this thread's own entries: no barrier needed
        const int p = min(tid + m * NTHREADS, PBLK - 1);
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        from[m] = tidx(kk, jj, ii);                      // where this thread's output elements sit in the tile
    }
    double cv[CPRE];
    __syncthreads();                                 // the box plan is complete; the plan has left the staging area
#pragma unroll 1
    for (int v = v0; v < nvar; v += stride) {
        const double* base = zipped + (int64_t)v * nb * BLK;
        double pv[PLAN_FULL];
#pragma unroll
        for (int m = 0; m < PLAN_FULL; ++m) pv[m] = ldg(base, off[m]);
        commit<true, PLAN_FULL, PLAN_FULL>(tile, scratch, bi, fp, pv, cv, false, base, tid);
        __syncthreads();
        double* out = padded + ((int64_t)v * nb + b) * PBLK;
#pragma unroll
        for (int m = 0; m < PLAN_FULL; ++m) {
            const int p = tid + m * NTHREADS;
            if (p < PBLK) out[p] = tile[from[m]];
        }
        __syncthreads();                             // the tile and the staging area are free again
    }
}

// Level-ordered ghost fill, centred variant: launched once per level, coarsest first; `blocks` lists
// the blocks of that level.  Copies and injections as in k_unzip; boxes that come from a coarser
// leaf are interpolated from that leaf's padded block, which an earlier launch has written.
// SOURCES: only the source leaves are filled, into a compact array indexed by src_slot.
template <bool SOURCES>
__global__ __launch_bounds__(NTHREADS) void k_unzip_centred(DeviceTree tr, const int32_t* __restrict__ blocks, int nvar,
                                                            const double* __restrict__ zipped, double* padded)
{
    __shared__ double tile[TILE];
    __shared__ double scratch[CENTRED_STAGING];
    __shared__ BlockInfo bi;
    static_assert(PLAN_FULL * NTHREADS * sizeof(uint32_t) <= CENTRED_STAGING * sizeof(double), "the plan is built in the staging area");
    const int tid = threadIdx.x;
    // workgroup r + G q: variables r, r + G, ... of the q-th block of the list, G = min(8, nvar), as in k_unzip
    const int stride = nvar < NXCD ? nvar : NXCD;
    const int64_t q = blockIdx.x / stride, b = blocks[q], nb = tr.nb;
    const int v0 = (int)(blockIdx.x - q * stride);
    const int64_t nout = SOURCES ? tr.n_src : nb;
    load_block_info(bi, tr, b, tid);
    __syncthreads();
    if (tid == 0) make_box_plan(bi);
    FillPlan<PLAN_FULL> fp;
    fp.src = reinterpret_cast<uint32_t*>(scratch);   // the staging area is free until the first interpolation
    make_plan_zipped<PLAN_FULL, PBLK>(fp, bi, tid);
    uint32_t off[PLAN_FULL];
    int from[PLAN_FULL];
#pragma unroll
    for (int m = 0; m < PLAN_FULL; ++m) {
        off[m] = fp.src[m * NTHREADS + tid];
        const int p = min(tid + m * NTHREADS, PBLK - 1);
        const int ii = p % NP, jj = (p / NP) % NP, kk = p / (NP * NP);
        from[m] = tidx(kk, jj, ii);
    }
    double cv[CPRE];
    const int64_t oslot = SOURCES ? (int64_t)tr.src_slot[b] : b;
    __syncthreads();                                 // the box plan is complete; the plan has left the staging area
#pragma unroll 1
    for (int v = v0; v < nvar; v += stride) {
        const double* base = zipped + (int64_t)v * nb * BLK;
        double pv[PLAN_FULL];
#pragma unroll
        for (int m = 0; m < PLAN_FULL; ++m) pv[m] = ldg(base, off[m]);
        commit<false, PLAN_FULL, PLAN_FULL>(tile, scratch, bi, fp, pv, cv, false, base, tid);   // stores only
        if (SOURCES) interp_boxes_centred<false>(tile, scratch, bi, padded + (int64_t)v * nout * PBLK, tid);
        else interp_boxes_centred<true>(tile, scratch, bi, padded + (int64_t)v * nout * PBLK, tid);
        __syncthreads();
        double* out = padded + ((int64_t)v * nout + oslot) * PBLK;
#pragma unroll
        for (int m = 0; m < PLAN_FULL; ++m) {
            const int p = tid + m * NTHREADS;
            if (p < PBLK) out[p] = tile[from[m]];
        }
        __syncthreads();                             // the tile and the staging area are free again
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

template <int KIND, bool ZIN, int EPI, bool CENTRED = false>
hipError_t launch_one(const DeviceTree& t, const RhsArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL((k_rhs<KIND, ZIN, EPI, CENTRED>), dim3(grid_for_blocks(t.nb)), dim3(NTHREADS), 0, s, t, a);
    return hipGetLastError();
}

template <int KIND>
hipError_t launch_kind(const DeviceTree& t, bool zin, bool centred, Epilogue ep, const RhsArgs& a, hipStream_t s)
{
    if (centred) {
        if (!zin || !a.pad_src) return hipErrorInvalidValue;
        switch (ep) {
        case kOutZipped: return launch_one<KIND, true, kOutZipped, true>(t, a, s);
        case kRkFirst: return launch_one<KIND, true, kRkFirst, true>(t, a, s);
        case kRkMiddle: return launch_one<KIND, true, kRkMiddle, true>(t, a, s);
        case kRkLast: return launch_one<KIND, true, kRkLast, true>(t, a, s);
        default: return hipErrorInvalidValue;
        }
    }
    if (!zin) {
        switch (ep) {
        case kOutPadded: return launch_one<KIND, false, kOutPadded>(t, a, s);
        case kOutZipped: return launch_one<KIND, false, kOutZipped>(t, a, s);
        case kRkFirst: return launch_one<KIND, false, kRkFirst>(t, a, s);
        case kRkMiddle: return launch_one<KIND, false, kRkMiddle>(t, a, s);
        case kRkLast: return launch_one<KIND, false, kRkLast>(t, a, s);
        default: return hipErrorInvalidValue;
        }
    }
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
    hipLaunchKernelGGL(k_unzip, dim3((unsigned)(t.nb * (nvar < NXCD ? nvar : NXCD))), dim3(NTHREADS), 0, s, t, nvar, zipped, padded);
    return hipGetLastError();
}

hipError_t launch_unzip_centred(const DeviceTree& t, const int64_t* level_start, bool sources_only, int nvar,
                                const double* zipped, double* padded, hipStream_t s)
{
    if (t.nb <= 0 || nvar <= 0) return hipSuccess;
    for (int l = 0; l < 20; ++l) {                   // coarsest level first; the stream orders the launches
        const int64_t n = level_start[l + 1] - level_start[l];
        if (n <= 0) continue;
        if (sources_only)
            hipLaunchKernelGGL(k_unzip_centred<true>, dim3((unsigned)(n * (nvar < NXCD ? nvar : NXCD))), dim3(NTHREADS), 0, s, t,
                               t.src_by_level + level_start[l], nvar, zipped, padded);
        else
            hipLaunchKernelGGL(k_unzip_centred<false>, dim3((unsigned)(n * (nvar < NXCD ? nvar : NXCD))), dim3(NTHREADS), 0, s, t,
                               t.by_level + level_start[l], nvar, zipped, padded);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_zip(const DeviceTree& t, int nvar, const double* padded, double* zipped, hipStream_t s)
{
    const int64_t n = t.nb * nvar;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_zip, dim3((unsigned)n), dim3(NTHREADS), 0, s, n, padded, zipped);
    return hipGetLastError();
}

hipError_t launch_rhs(const DeviceTree& t, ot_rhs_kind kind, bool in_zipped, bool centred, Epilogue ep, const RhsArgs& args,
                      hipStream_t s)
{
    if (t.nb <= 0) return hipSuccess;
    switch (kind) {
    case OT_RHS_DERIVS: return launch_kind<OT_RHS_DERIVS>(t, in_zipped, centred, ep, args, s);
    case OT_RHS_WAVE: return launch_kind<OT_RHS_WAVE>(t, in_zipped, centred, ep, args, s);
    case OT_RHS_BURGERS: return launch_kind<OT_RHS_BURGERS>(t, in_zipped, centred, ep, args, s);
    case OT_RHS_SYN24: return launch_kind<OT_RHS_SYN24>(t, in_zipped, centred, ep, args, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace octfd
