// Host-only check of the derived tables of the library's tree (no GPU, no HIP call): the virtual blocks with the
// ghost table that names them, and the sibling pairs.  Built with g++ together with csrc/octree_host.cpp by tests/test_library_host.py.
#include <cmath>
#include <cstdio>
#include <vector>

#include "kernels.hpp"
#include "octree_host.hpp"

using namespace octfd;

static int fail(const char* what, long b) { std::printf("FAILED: %s (block %ld)\n", what, b); return 1; }

static int check(const HostTree& t)
{
    const long nb = static_cast<long>(t.leaves.size());
    // virtual blocks: every coarser entry of the ghost table has become a virtual block that is the right child
    // octant of the right source leaf; every virtual block is used, listed once per level, one level below its source
    const long nv = static_cast<long>(t.n_virt);
    if (static_cast<long>(t.vblk.size()) != 2 * nv || static_cast<long>(t.vlist.size()) != nv || t.ghost_v.size() != t.ghost.size())
        return fail("sizes of the virtual-block tables", -1);
    std::vector<int> used(nv, 0);
    for (long b = 0; b < nb; ++b)
        for (int dir = 0; dir < kDirs; ++dir) {
            const int32_t* e = &t.ghost[(b * kDirs + dir) * kEntry];
            const int32_t* v = &t.ghost_v[(b * kDirs + dir) * kEntry];
            if (e[0] != kCoarser) {
                for (int m = 0; m < kEntry; ++m)
                    if (e[m] != v[m]) return fail("an entry that is not coarser was changed", b);
                continue;
            }
            if (v[0] != kVirtual || v[1] < 0 || v[1] >= nv) return fail("a coarser entry is not a virtual block", b);
            const ot_leaf& o = t.leaves[b];
            const uint32_t mask = (1u << o.level) - 1;
            const uint32_t x = (o.ix + (dir % 3 - 1)) & mask, y = (o.iy + ((dir / 3) % 3 - 1)) & mask, z = (o.iz + (dir / 9 - 1)) & mask;
            const ot_leaf& src = t.leaves[t.vblk[2 * v[1]]];
            if (t.vblk[2 * v[1]] != e[1]) return fail("source leaf of a virtual block", b);
            if (src.level + 1 != o.level || src.ix != x >> 1 || src.iy != y >> 1 || src.iz != z >> 1) return fail("a virtual block is not inside its source leaf", b);
            if (t.vblk[2 * v[1] + 1] != static_cast<int32_t>((x & 1) | ((y & 1) << 1) | ((z & 1) << 2))) return fail("child octant of a virtual block", b);
            ++used[v[1]];
        }
    // the rows and planes of a virtual block that the fill writes are exactly those that some ghost point of some
    // block lies in: walk every ghost point of every padded block
    if (static_cast<long>(t.vneed.size()) != nv) return fail("size of the table of needed rows", -1);
    std::vector<int32_t> seen(nv, 0);
    for (long b = 0; b < nb; ++b)
        for (int kk = 0; kk < 14; ++kk)
            for (int jj = 0; jj < 14; ++jj)
                for (int ii = 0; ii < 14; ++ii) {
                    const int r[3] = {ii < 3 ? 0 : (ii < 11 ? 1 : 2), jj < 3 ? 0 : (jj < 11 ? 1 : 2), kk < 3 ? 0 : (kk < 11 ? 1 : 2)};
                    const int32_t* v = &t.ghost_v[(b * kDirs + r[2] * 9 + r[1] * 3 + r[0]) * kEntry];
                    if (v[0] != kVirtual) continue;
                    // position inside the neighbour in that direction
                    const int ly = jj - 3 + (1 - r[1]) * 8, lz = kk - 3 + (1 - r[2]) * 8;
                    if (ly < 0 || ly > 7 || lz < 0 || lz > 7) return fail("position inside a virtual block", b);
                    seen[v[1]] |= 1 << ly | 1 << (8 + lz);
                }
    long written = 0;
    for (long v = 0; v < nv; ++v) {
        if (t.vneed[v] != seen[v]) return fail("rows and planes of a virtual block that are read", v);
        written += 8 * __builtin_popcount(seen[v] & 0xFF) * __builtin_popcount(seen[v] >> 8);
    }
    if (nv) std::printf("points of the virtual blocks that are written: %.1f %%\n", 100.0 * written / (512.0 * nv));
    std::vector<int> listed(nv, 0);
    for (int l = 0; l < 20; ++l) {
        if (t.vlevel_start[l] > t.vlevel_start[l + 1]) return fail("level ranges of the virtual blocks", l);
        for (int64_t q = t.vlevel_start[l]; q < t.vlevel_start[l + 1]; ++q) {
            const int32_t v = t.vlist[q];
            if (v < 0 || v >= nv || static_cast<int>(t.leaves[t.vblk[2 * v]].level) + 1 != l) return fail("level of a listed virtual block", v);
            ++listed[v];
        }
    }
    if (t.vlevel_start[0] != 0 || t.vlevel_start[20] != nv) return fail("level ranges do not cover the virtual blocks", -1);
    for (long v = 0; v < nv; ++v) {
        if (!used[v]) return fail("a virtual block that nobody reads", v);
        if (listed[v] != 1) return fail("a virtual block is not listed exactly once", v);
        if (v > 0 && (t.vblk[2 * v] < t.vblk[2 * v - 2] || (t.vblk[2 * v] == t.vblk[2 * v - 2] && t.vblk[2 * v + 1] <= t.vblk[2 * v - 1])))
            return fail("order of the virtual blocks", v);
    }
    // work units of the two-block kernel: every block exactly once, in Morton order; a pair is the lower and upper x
    // child of one parent, a single block has no leaf as x sibling
    std::vector<int> times(nb, 0);
    long npairs = 0, nsingles = 0, last = -1;
    for (int32_t u : t.units) {
        const long b = u & ~kUnitSingle;
        if (b < 0 || b >= nb || b <= last) return fail("unit id or order", b);
        last = b;
        ++times[b];
        const ot_leaf& o = t.leaves[b];
        if (u & kUnitSingle) {
            ++nsingles;
            const long sib = (o.ix & 1) ? b - 1 : b + 1;
            if (sib >= 0 && sib < nb) {
                const ot_leaf& n = t.leaves[sib];
                if (n.level == o.level && (n.ix ^ 1) == o.ix && n.iy == o.iy && n.iz == o.iz) return fail("a single block has a leaf as x sibling", b);
            }
        } else {
            ++npairs;
            if (b + 1 >= nb) return fail("pair id", b);
            const ot_leaf& hi = t.leaves[b + 1];
            if ((o.ix & 1) || hi.level != o.level || hi.ix != o.ix + 1 || hi.iy != o.iy || hi.iz != o.iz) return fail("not an x-sibling pair", b);
            ++times[b + 1];
        }
    }
    for (long b = 0; b < nb; ++b)
        if (times[b] != 1) return fail("a block is not covered exactly once by the units", b);
    std::printf("blocks %ld, virtual blocks %ld, pairs %ld, singles %ld\n", nb, nv, npairs, nsingles);
    return 0;
}

int main()
{
    // an adaptive tree with two centres (levels 3..6), a uniform one, and one centre near the periodic corner
    const uint32_t pts[6] = {416961, 715879, 415070, 444683, 374201, 590464};
    const uint32_t rad[3] = {125829, 125829, 125829};
    HostTree a, u, c;
    ot_build_params p{3, 6, 2, pts, rad, 8, 3, 1};
    if (build_tree(p, a) != OT_OK || check(a)) return 1;
    ot_build_params q{4, 4, 0, nullptr, nullptr, 8, 3, 1};
    if (build_tree(q, u) != OT_OK || check(u)) return 1;
    const uint32_t corner[3] = {1000, 2000, 1040000};
    const uint32_t rad2[2] = {50000, 60000};
    ot_build_params r{3, 5, 1, corner, rad2, 8, 3, 1};
    if (build_tree(r, c) != OT_OK || check(c)) return 1;
    return 0;
}
