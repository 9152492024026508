// Launch interface between the C ABI (capi.cpp) and the gfx950 kernels (kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "octfd.h"

namespace octfd {

struct DeviceTree {
    const ot_leaf* leaves;   // [nb]
    const int32_t* ghost;    // [nb][27][5]
    const int32_t* coarse;   // [nb][32] coarser sources with their boxes, and coarser faces (see HostTree)
    const int32_t* by_level; // [nb] block ids sorted by level
    int64_t nb;
    // centred ghost rule: the leaves that are a coarser source of some block ("source leaves")
    const int32_t* src_slot;     // [nb] position of a source leaf in a compact padded array, -1 for the others
    const int32_t* src_by_level; // [n_src] ids of the source leaves sorted by level
    int64_t n_src;
    const int32_t* sched;        // [n_sched] launch order of the 24-field kernel, see HostTree::sched
    int64_t n_sched;
    // virtual blocks (see HostTree): the ghost table that names them, and the source leaves they are children of
    const int32_t* ghost_v;      // [nb][27][5]
    const int32_t* vsrc;         // [n_src][3] {leaf id, mask of child octants, first virtual block}
    const int32_t* vblk;         // [n_virt][2] {source leaf, child octant} of every virtual block
    int64_t n_virt;
    // the 24-field system on zipped input: sibling pairs (first block of each) for the two-block kernel, and the
    // remaining blocks, which run the one-block kernel
    const int32_t* pairs;
    int64_t n_pairs;
    const int32_t* singles;
    int64_t n_singles;
};

// HostTree::sched is made of chunks of this many entries; the kernels hand one chunk to one XCD
constexpr int kSchedChunk = 16;
constexpr int kSchedXcds = 8;    // XCDs of the device: workgroup i runs on XCD i mod 8
constexpr int32_t kSchedCoarse = 1 << 30;   // flag on a schedule entry: the block has a coarser source

// how the right-hand side leaves the kernel
enum Epilogue : int {
    kOutPadded = 0,   // interior of a padded-shaped array
    kOutZipped = 1,   // zipped array
    kRkFirst = 2,     // acc = k;        stage = fma(c, k, u)        (u is the kernel's input)
    kRkMiddle = 3,    // acc = acc + 2k; stage = fma(c, k, u)
    kRkLast = 4       // u = fma(c, acc + k, u)
};

struct RhsArgs {
    const double* in;   // padded [V][nb][2744] or zipped [V][nb][512]
    double* out;        // kOutPadded / kOutZipped: result; kRkFirst / kRkMiddle: next stage vector
    double* acc;        // Runge-Kutta accumulator (zipped)
    double* u;          // state at the start of the step (zipped); written by kRkLast
    const double* pad_src;   // centred ghost rule only: padded blocks of the source leaves of `in`, [V][n_src][2744]
    const double* virt;      // the virtual blocks of `in`, [V][n_virt][512] (kernels that read ghost_v; filled by launch_virtual)
    double* stash;      // SYN24 only: array shaped like `out` whose variables 10..19 may be used as
                        // scratch until their final values are written (may be `out` itself)
    double c;           // dt/2, dt or dt/6
    double sigma;       // Kreiss-Oliger strength
};

hipError_t launch_unzip(const DeviceTree& t, int nvar, const double* zipped, double* padded, hipStream_t s);
// level-ordered ghost fill with centred coarse-lattice stencils; level_start[21] as in HostTree.
// sources_only = false: every block, padded [nvar][nb][2744];  true: only the source leaves (level_start
// then refers to src_by_level), padded [nvar][n_src][2744] indexed by src_slot
hipError_t launch_unzip_centred(const DeviceTree& t, const int64_t* level_start, bool sources_only, int nvar,
                                const double* zipped, double* padded, hipStream_t s);
// fills the virtual blocks of a zipped array: virt [nvar][n_virt][512], each the child octant of its source leaf,
// every point interpolated inside that leaf exactly as a ghost point is in unzip
hipError_t launch_virtual(const DeviceTree& t, int nvar, const double* zipped, double* virt, hipStream_t s);
hipError_t launch_zip(const DeviceTree& t, int nvar, const double* padded, double* zipped, hipStream_t s);
// the 24-field right-hand side on the sibling pairs of the tree (pair.hip): zipped input with its virtual blocks,
// epilogue kOutZipped or one of the Runge-Kutta stages
hipError_t launch_rhs_pairs(const DeviceTree& t, Epilogue ep, const RhsArgs& args, const int32_t* pairs, int64_t npairs, hipStream_t s);
// in_zipped = false: args.in is padded; true: args.in is zipped.  centred (zipped input only): ghost
// values from coarser leaves follow the centred rule and are read from args.pad_src
hipError_t launch_rhs(const DeviceTree& t, ot_rhs_kind kind, bool in_zipped, bool centred, Epilogue ep,
                      const RhsArgs& args, hipStream_t s);

}  // namespace octfd
