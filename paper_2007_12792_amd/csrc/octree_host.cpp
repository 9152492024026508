// Host octree engine: refinement, 26-neighbour periodic 2:1 balance, Morton ordering and the
// ghost-source table (see octfd.h, octree_build).  The tree is an explicit pointer octree; the
// eight children of a node are stored contiguously in Morton child order c = (cz<<2)|(cy<<1)|cx,
// so a depth-first walk visits the leaves in storage order and neighbours are found by descending
// from the root.
#include "octree_host.hpp"

#include "kernels.hpp"

#include <deque>

namespace octfd {
namespace {

constexpr int kQBits = 20;
constexpr int32_t kLeaf = -1, kUnset = -2;

struct Node {
    int32_t first_child;  // >= 0 internal, kLeaf, or kUnset (from_leaves: nothing placed here yet)
    uint32_t level, ix, iy, iz;
    int32_t leaf_id;
};

struct Octree {
    std::vector<Node> nodes;

    Octree() { nodes.push_back(Node{kLeaf, 0, 0, 0, 0, -1}); }

    // turn node n into an internal node with eight children in state `child_state`
    int32_t split(int32_t n, int32_t child_state = kLeaf)
    {
        const Node p = nodes[n];
        const int32_t first = static_cast<int32_t>(nodes.size());
        for (uint32_t c = 0; c < 8; ++c)
            nodes.push_back(Node{child_state, p.level + 1, 2 * p.ix + (c & 1), 2 * p.iy + ((c >> 1) & 1),
                                 2 * p.iz + ((c >> 2) & 1), -1});
        nodes[n].first_child = first;
        return first;
    }

    static uint32_t child_slot(uint32_t l, uint32_t x, uint32_t y, uint32_t z, uint32_t node_level)
    {
        const uint32_t sh = l - node_level - 1;
        return (((z >> sh) & 1) << 2) | (((y >> sh) & 1) << 1) | ((x >> sh) & 1);
    }

    // deepest existing node on the path from the root towards octant (l; x, y, z), depth <= l
    int32_t descend(uint32_t l, uint32_t x, uint32_t y, uint32_t z) const
    {
        int32_t n = 0;
        while (nodes[n].first_child >= 0 && nodes[n].level < l)
            n = nodes[n].first_child + static_cast<int32_t>(child_slot(l, x, y, z, nodes[n].level));
        return n;
    }
};

// periodic distance (2^20-lattice units) from coordinate c to the closed interval [lo, lo+s]
inline int64_t periodic_gap(int64_t c, int64_t lo, int64_t s)
{
    constexpr int64_t kOne = int64_t(1) << kQBits;
    const int64_t t = ((c - lo) % kOne + kOne) % kOne;  // offset of c past lo, going upwards
    if (t <= s) return 0;
    const int64_t up = t - s, down = kOne - t;
    return up < down ? up : down;
}

bool near_seed(const Node& o, const ot_build_params& p)
{
    const int64_t s = int64_t(1) << (kQBits - o.level);
    const int64_t R = p.radius_q20[o.level - p.lmin];
    const int64_t a[3] = {o.ix, o.iy, o.iz};
    for (uint32_t q = 0; q < p.npts; ++q) {
        int64_t d2 = 0;
        for (int d = 0; d < 3; ++d) {
            const int64_t g = periodic_gap(p.pts_q20[3 * q + d], a[d] * s, s);
            d2 += g * g;
        }
        if (d2 < R * R) return true;
    }
    return false;
}

// Every leaf on the queue makes sure that none of its 26 neighbours is more than one level
// coarser.  Splitting a leaf can only create new obligations for its own children, so they are
// queued; leaves that were already checked stay valid because neighbours only ever get finer.
void balance(Octree& t, std::deque<int32_t>& queue)
{
    while (!queue.empty()) {
        const int32_t n = queue.front();
        queue.pop_front();
        if (t.nodes[n].first_child != kLeaf) continue;
        const Node o = t.nodes[n];
        if (o.level < 2) continue;
        const uint32_t mask = (1u << o.level) - 1;
        for (int dz = -1; dz <= 1; ++dz)
            for (int dy = -1; dy <= 1; ++dy)
                for (int dx = -1; dx <= 1; ++dx) {
                    if (!dx && !dy && !dz) continue;
                    const uint32_t x = (o.ix + dx) & mask, y = (o.iy + dy) & mask, z = (o.iz + dz) & mask;
                    for (;;) {
                        const int32_t m = t.descend(o.level, x, y, z);
                        if (t.nodes[m].first_child != kLeaf || t.nodes[m].level + 1 >= o.level) break;
                        const int32_t first = t.split(m);
                        for (int c = 0; c < 8; ++c) queue.push_back(first + c);
                    }
                }
    }
}

void emit_leaves(Octree& t, int32_t n, std::vector<ot_leaf>& out)
{
    Node& o = t.nodes[n];
    if (o.first_child == kLeaf) {
        o.leaf_id = static_cast<int32_t>(out.size());
        out.push_back(ot_leaf{o.level, o.ix, o.iy, o.iz});
        return;
    }
    const int32_t first = o.first_child;
    for (int c = 0; c < 8; ++c) emit_leaves(t, first + c, out);
}

// Ghost-source table.  Returns OT_OK or OT_E_UNBALANCED.
int make_ghost_table(const Octree& t, const std::vector<ot_leaf>& leaves, std::vector<int32_t>& ghost)
{
    const size_t nb = leaves.size();
    ghost.assign(nb * kDirs * kEntry, -1);
    for (size_t b = 0; b < nb; ++b) {
        const ot_leaf& o = leaves[b];
        const uint32_t mask = (1u << o.level) - 1;
        for (int dir = 0; dir < kDirs; ++dir) {
            const int d[3] = {dir % 3 - 1, (dir / 3) % 3 - 1, dir / 9 - 1};
            int32_t* e = &ghost[(b * kDirs + dir) * kEntry];
            const uint32_t x = (o.ix + d[0]) & mask, y = (o.iy + d[1]) & mask, z = (o.iz + d[2]) & mask;
            const int32_t m = t.descend(o.level, x, y, z);
            const Node& nd = t.nodes[m];
            if (nd.first_child == kLeaf) {
                if (nd.level == o.level) e[0] = kSame;
                else if (nd.level + 1 == o.level) e[0] = kCoarser;
                else return OT_E_UNBALANCED;
                e[1] = nd.leaf_id;
                continue;
            }
            // the neighbouring octant is subdivided: take the children that touch this block.
            // Along an axis with d = -1 they are the upper children, with d = +1 the lower ones;
            // axes with d = 0 are free and enumerated x, then y, then z (ascending Morton order).
            e[0] = kFiner;
            int nfree = 0, free_axis[3];
            for (int ax = 0; ax < 3; ++ax) if (d[ax] == 0) free_axis[nfree++] = ax;
            for (int q = 0; q < (1 << nfree); ++q) {
                int bit[3];
                for (int ax = 0; ax < 3; ++ax) bit[ax] = d[ax] < 0 ? 1 : 0;
                for (int f = 0; f < nfree; ++f) bit[free_axis[f]] = (q >> f) & 1;
                const Node& ch = t.nodes[nd.first_child + ((bit[2] << 2) | (bit[1] << 1) | bit[0])];
                if (ch.first_child != kLeaf) return OT_E_UNBALANCED;
                e[1 + q] = ch.leaf_id;
            }
        }
    }
    return OT_OK;
}

}  // namespace

void make_virtual_blocks(HostTree& t)
{
    const size_t nb = t.leaves.size();
    // which child octant of its parent the neighbour octant in direction dir is: the low bit of its anchor
    auto octant_of = [&](size_t b, int dir) {
        const ot_leaf& o = t.leaves[b];
        const uint32_t x = o.ix + (dir % 3 - 1), y = o.iy + ((dir / 3) % 3 - 1), z = o.iz + (dir / 9 - 1);   // mod 2^l keeps the low bit
        return static_cast<int>((x & 1) | ((y & 1) << 1) | ((z & 1) << 2));
    };
    // per leaf: which of its child octants some block needs
    std::vector<uint8_t> mask(nb, 0);
    for (size_t b = 0; b < nb; ++b)
        for (int dir = 0; dir < kDirs; ++dir) {
            const int32_t* e = &t.ghost[(b * kDirs + dir) * kEntry];
            if (e[0] == kCoarser) mask[e[1]] |= static_cast<uint8_t>(1 << octant_of(b, dir));
        }
    // numbered by source leaf, then octant
    std::vector<int32_t> first(nb, 0);
    t.vblk.clear();
    int32_t n = 0;
    for (size_t s = 0; s < nb; ++s) {
        first[s] = n;
        for (int c = 0; c < 8; ++c)
            if ((mask[s] >> c) & 1) {
                t.vblk.push_back(static_cast<int32_t>(s));
                t.vblk.push_back(c);
                ++n;
            }
    }
    t.n_virt = n;
    // by level
    int64_t count[21] = {};
    for (int32_t q = 0; q < n; ++q) ++count[t.leaves[t.vblk[2 * q]].level + 2];      // its own level + 1
    for (int l = 1; l <= 20; ++l) count[l] += count[l - 1];
    for (int l = 0; l <= 20; ++l) t.vlevel_start[l] = count[l];
    t.vlist.assign(n, 0);
    for (int32_t q = 0; q < n; ++q) t.vlist[count[t.leaves[t.vblk[2 * q]].level + 1]++] = q;
    t.ghost_v = t.ghost;
    t.vneed.assign(n, 0);
    // a block reads, of its neighbour in direction d, the three layers next to itself along every axis with d != 0
    // and all eight along the others
    auto layers = [](int d) { return d > 0 ? 0x07 : (d < 0 ? 0xE0 : 0xFF); };
    for (size_t b = 0; b < nb; ++b)
        for (int dir = 0; dir < kDirs; ++dir) {
            int32_t* e = &t.ghost_v[(b * kDirs + dir) * kEntry];
            if (e[0] != kCoarser) continue;
            const int c = octant_of(b, dir);
            const int32_t src = e[1];
            e[0] = kVirtual;
            e[1] = first[src] + __builtin_popcount(static_cast<unsigned>(mask[src]) & ((1u << c) - 1));
            t.vneed[e[1]] |= layers((dir / 3) % 3 - 1) | layers(dir / 9 - 1) << 8;
        }
}

void make_units(HostTree& t)
{
    const size_t nb = t.leaves.size();
    t.units.clear();
    for (size_t b = 0; b < nb;) {
        const ot_leaf& o = t.leaves[b];
        if (b + 1 < nb && !(o.ix & 1)) {
            const ot_leaf& n = t.leaves[b + 1];
            if (n.level == o.level && n.ix == o.ix + 1 && n.iy == o.iy && n.iz == o.iz) {
                t.units.push_back(static_cast<int32_t>(b));
                b += 2;
                continue;
            }
        }
        t.units.push_back(static_cast<int32_t>(b) | kUnitSingle);
        ++b;
    }
}

int build_tree(const ot_build_params& p, HostTree& out)
{
    if (p.lmin < 3 || p.lmax < p.lmin || p.lmax > 19) return OT_E_BADARG;
    if (p.points_per_dim != 8 || p.pad != 3 || p.periodic != 1) return OT_E_UNSUPPORTED;
    if (p.npts && !p.pts_q20) return OT_E_BADARG;
    if (p.lmax > p.lmin && !p.radius_q20) return OT_E_BADARG;
    for (uint32_t q = 0; q < 3 * p.npts; ++q)
        if (p.pts_q20[q] >> kQBits) return OT_E_BADARG;
    // no two points of the periodic cube are further apart than sqrt(3) * 2^19 lattice units; larger radii say
    // nothing more, and beyond 2^31.5 their square would overflow the 64-bit comparison in near_seed()
    for (uint32_t l = p.lmin; l < p.lmax; ++l)
        if (p.radius_q20[l - p.lmin] > (2u << kQBits)) return OT_E_BADARG;

    Octree t;
    std::deque<int32_t> work{0};
    std::deque<int32_t> leaves_to_balance;
    // uniform refinement to lmin, then seed-driven refinement; each node is visited once
    while (!work.empty()) {
        const int32_t n = work.front();
        work.pop_front();
        const Node o = t.nodes[n];
        const bool grow = o.level < p.lmin || (o.level < p.lmax && near_seed(o, p));
        if (!grow) { leaves_to_balance.push_back(n); continue; }
        const int32_t first = t.split(n);
        for (int c = 0; c < 8; ++c) work.push_back(first + c);
    }
    balance(t, leaves_to_balance);
    out.leaves.clear();
    emit_leaves(t, 0, out.leaves);
    const int rc = make_ghost_table(t, out.leaves, out.ghost);
    if (rc == OT_OK) { make_virtual_blocks(out); make_units(out); }
    return rc;
}

int tree_from_leaves(const ot_leaf* leaves, size_t n, HostTree& out)
{
    if (!leaves || n == 0) return OT_E_BADARG;
    Octree t;
    t.nodes[0].first_child = kUnset;
    for (size_t i = 0; i < n; ++i) {
        const ot_leaf& o = leaves[i];
        if (o.level < 3 || o.level > 19 || (o.ix >> o.level) || (o.iy >> o.level) || (o.iz >> o.level))
            return OT_E_BADARG;
        int32_t m = 0;
        while (t.nodes[m].level < o.level) {
            if (t.nodes[m].first_child == kLeaf) return OT_E_INCOMPLETE;      // inside another leaf
            if (t.nodes[m].first_child == kUnset) t.split(m, kUnset);
            m = t.nodes[m].first_child + static_cast<int32_t>(Octree::child_slot(o.level, o.ix, o.iy, o.iz, t.nodes[m].level));
        }
        if (t.nodes[m].first_child != kUnset) return OT_E_INCOMPLETE;        // duplicate or ancestor of a leaf
        t.nodes[m].first_child = kLeaf;
    }
    for (const Node& nd : t.nodes)
        if (nd.first_child == kUnset) return OT_E_INCOMPLETE;                // a gap
    out.leaves.clear();
    emit_leaves(t, 0, out.leaves);
    const int rc = make_ghost_table(t, out.leaves, out.ghost);
    if (rc == OT_OK) { make_virtual_blocks(out); make_units(out); }
    return rc;
}

}  // namespace octfd
