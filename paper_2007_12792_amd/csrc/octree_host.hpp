// Host-side octree engine of liboctfd: pointer octree, queue-driven 2:1 balance, Morton-order
// traversal and the ghost-source table.  No device code here.
#pragma once
#include <cstdint>
#include <vector>

#include "octfd.h"

namespace octfd {

constexpr int kDirs = 27;          // directions (dz+1)*9 + (dy+1)*3 + (dx+1)
constexpr int kEntry = 5;          // {kind, id0..id3}
enum GhostKind : int32_t { kSame = 0, kFiner = 1, kCoarser = 2, kVirtual = 3 };

struct HostTree {
    std::vector<ot_leaf> leaves;   // Morton order
    std::vector<int32_t> ghost;    // [nb][27][5]
    // "Virtual blocks".  Where the same-level neighbour octant of a block does not exist because its parent L is
    // a leaf, the ghost values in that direction are interpolated inside L, and what they are depends only on L's
    // data and on the fine position inside L, not on which block asks.  Such an octant can therefore be filled
    // once, like a child of L ("virtual block"), after which the blocks around it read it
    // exactly like a neighbour of their own level.
    //   vblk    [n_virt][2]        per virtual block {source leaf id, child octant (ox | oy<<1 | oz<<2)}, ordered by
    //                              source leaf (Morton order), then octant
    //   ghost_v [nb][27][5]        the ghost table with every coarser entry replaced by {kVirtual, virtual block}
    //   n_virt                     number of virtual blocks
    //   vlist   [n_virt]           virtual blocks sorted by level (the level of a virtual block is its source leaf's
    //                              plus one): level l occupies vlist[vlevel_start[l] .. vlevel_start[l+1]).  With the
    //                              centred ghost rule a level's virtual blocks read those of the level before.
    //   vneed   [n_virt]           which y rows (bits 0..7) and z planes (bits 8..15) of a virtual block any block reads: the
    //                              union, per axis, over the blocks that have it as a neighbour.  The fill writes only
    //                              those (whole x rows of them); the rest of a virtual block is never read.
    std::vector<int32_t> vblk, ghost_v, vlist, vneed;
    int64_t n_virt = 0;
    int64_t vlevel_start[21] = {};
    // Work units of the two-block kernel of the 24-field system, in Morton order: the first block of every two
    // leaves that are the lower and upper x child of one parent (they follow each other in storage), and, flagged
    // with kUnitSingle, every other block (a leaf whose x sibling is subdivided).  Every block belongs to exactly one unit.
    std::vector<int32_t> units;
};

// Each returns an OT_* status.
int build_tree(const ot_build_params& p, HostTree& out);
int tree_from_leaves(const ot_leaf* leaves, size_t n, HostTree& out);
void make_virtual_blocks(HostTree& t);
void make_units(HostTree& t);

}  // namespace octfd
