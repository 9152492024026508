// Host-side octree engine of liboctfd: pointer octree, queue-driven 2:1 balance, Morton-order
// traversal and the ghost-source table.  No device code here.
#pragma once
#include <cstdint>
#include <vector>

#include "octfd.h"

namespace octfd {

constexpr int kDirs = 27;          // directions (dz+1)*9 + (dy+1)*3 + (dx+1)
constexpr int kEntry = 5;          // {kind, id0..id3}
constexpr int kCoarseRow = 32;     // ints per block in HostTree::coarse
enum GhostKind : int32_t { kSame = 0, kFiner = 1, kCoarser = 2, kVirtual = 3 };
constexpr int kVsrcRow = 3;        // ints per source leaf in HostTree::vsrc

struct HostTree {
    std::vector<ot_leaf> leaves;   // Morton order
    std::vector<int32_t> ghost;    // [nb][27][5]
    // Derived from `ghost` for the kernels, kCoarseRow ints per block:
    //   [0..15]  the distinct coarser source leaves, each with the box of the padded block it covers:
    //            8 x {leaf id, packed ranges}, id -1 ends the list; packed = xlo | xhi<<2 | ylo<<4 |
    //            yhi<<6 | zlo<<8 | zhi<<10 with 0/1/2 naming the ghost-low, interior and ghost-high
    //            part of an axis (inclusive ranges);
    //            Sources whose box is a single corner of the padded block come last;
    //   [16]     number of face neighbours that are coarser, then [17..28] that many {face, leaf id}
    //            pairs, face = 2*axis + (0 low side, 1 high side);
    //   [29]     number of sources in front of the corner-only ones.
    // Read by the kernels that write padded blocks (unzip, unzip_centred).
    std::vector<int32_t> coarse;
    // Block ids sorted by level (ascending, Morton order within a level): blocks of level l are
    // by_level[level_start[l] .. level_start[l+1]).  Used by the level-ordered ghost fill.
    std::vector<int32_t> by_level;
    int64_t level_start[21] = {};
    // "Source leaves": the leaves that some block takes ghost values from by coarse-to-fine
    // interpolation.  src_slot[b] numbers them (Morton order), -1 for all other leaves;
    // src_by_level / src_level_start list them by level like by_level / level_start.
    std::vector<int32_t> src_slot, src_by_level;
    int64_t src_level_start[21] = {};
    // "Virtual blocks".  Where the same-level neighbour octant of a block does not exist because its parent L is
    // a leaf, the ghost values in that direction are interpolated inside L, and what they are depends only on L's
    // data and on the fine position inside L, not on which block asks.  Such an octant can therefore be filled
    // once, all 8^3 points of it, like a child of L ("virtual block"), after which the blocks around it read it
    // exactly like a neighbour of their own level.
    //   vsrc    [n_src][kVsrcRow]  per source leaf, in Morton order: {leaf id, mask of the child octants
    //                              (bit ox | oy<<1 | oz<<2) that some block needs, index of its first virtual block};
    //                              a leaf's virtual blocks are numbered consecutively in ascending octant order
    //   vblk    [n_virt][2]        per virtual block {source leaf id, child octant}
    //   ghost_v [nb][27][5]        the ghost table with every coarser entry replaced by {kVirtual, virtual block}
    //   n_virt                     number of virtual blocks
    //   vlist   [n_virt]           virtual blocks sorted by level (the level of a virtual block is its source leaf's
    //                              plus one): level l occupies vlist[vlevel_start[l] .. vlevel_start[l+1]).  With the
    //                              centred ghost rule a level's virtual blocks read those of the level before.
    std::vector<int32_t> vsrc, vblk, ghost_v, vlist;
    int64_t n_virt = 0;
    int64_t vlevel_start[21] = {};
    // Sibling pairs for the two-block kernel of the 24-field system: `pairs` lists the first block of every two
    // leaves that are the lower and upper x child of one parent (they follow each other in Morton order), `singles`
    // every other block (a leaf whose x sibling is subdivided).  Both in Morton order; together they cover every
    // block exactly once.
    std::vector<int32_t> pairs, singles;
};

// Each returns an OT_* status.
int build_tree(const ot_build_params& p, HostTree& out);
int tree_from_leaves(const ot_leaf* leaves, size_t n, HostTree& out);
void make_coarse_sources(HostTree& t);
void make_level_lists(HostTree& t);
void make_virtual_blocks(HostTree& t);
void make_pairs(HostTree& t);

}  // namespace octfd
