// Launch interface between the C ABI (capi.cpp) and the gfx950 kernels (kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "octfd.h"

namespace octfd {

struct DeviceTree {
    const ot_leaf* leaves;   // [nb]
    int64_t nb;
    // virtual blocks (see HostTree): the ghost table that names them, what each is, and their order by level
    const int32_t* ghost_v;  // [nb][27][5]
    const int32_t* vblk;     // [n_virt][2] {source leaf, child octant} of every virtual block
    const int32_t* vlist;    // [n_virt] virtual blocks sorted by level
    int64_t n_virt;
    // the 24-field system on zipped input: the work units of the two-block kernel (see HostTree::units)
    const int32_t* units;
    int64_t n_units;
    const int32_t* vneed;    // [n_virt] y rows (bits 0..7) and z planes (bits 8..15) of a virtual block that are read at all
};

constexpr int32_t kUnitSingle = 1 << 30;   // flag on a unit: one block without a partner

// workgroup i runs on XCD i mod kXcds; the kernels deal chunks of kChunk consecutive blocks to the XCDs in turn
constexpr int kSchedChunk = 16;
constexpr int kSchedXcds = 8;

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
    const double* virt;      // zipped input: the virtual blocks of `in`, [V][n_virt][512], filled by launch_virtual or
                             // launch_virtual_centred (which of the two decides the ghost rule)
    double* stash;      // SYN24 only: array shaped like `out` whose variables 10..19 may be used as
                        // scratch until their final values are written (may be `out` itself)
    double c;           // dt/2, dt or dt/6
    double sigma;       // Kreiss-Oliger strength
};

// padded [nvar][nb][2744] from zipped and its virtual blocks (filled by one of the two calls below: which one decides
// the ghost rule)
hipError_t launch_unzip(const DeviceTree& t, int nvar, const double* zipped, const double* virt, double* padded, hipStream_t s);
// fills the virtual blocks of a zipped array: virt [nvar][n_virt][512], each the child octant of its source leaf,
// every point interpolated inside that leaf exactly as a ghost point is in unzip ...
hipError_t launch_virtual(const DeviceTree& t, int nvar, const double* zipped, double* virt, hipStream_t s);
// ... or in unzip_centred (level by level; vlevel_start[21] as in HostTree)
hipError_t launch_virtual_centred(const DeviceTree& t, const int64_t* vlevel_start, int nvar, const double* zipped, double* virt,
                                   hipStream_t s);
hipError_t launch_zip(const DeviceTree& t, int nvar, const double* padded, double* zipped, hipStream_t s);
// the 24-field right-hand side over the units of the tree (pair.hip): zipped input with its virtual blocks,
// epilogue kOutZipped or one of the Runge-Kutta stages
hipError_t launch_rhs_pairs(const DeviceTree& t, Epilogue ep, const RhsArgs& args, hipStream_t s);
// in_zipped = false: args.in is padded; true: args.in is zipped and args.virt holds its virtual blocks
hipError_t launch_rhs(const DeviceTree& t, ot_rhs_kind kind, bool in_zipped, Epilogue ep, const RhsArgs& args, hipStream_t s);

}  // namespace octfd
