// Inter-grid transfer after a regrid (see octfd.h, regrid_plan): host-side plan and the launch
// interface of its kernel.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "octfd.h"

namespace octfd {

enum TransferKind : int32_t { kCopy = 0, kProlong = 1, kInject = 2 };
constexpr int kTransferRow = 4;   // {kind, first source leaf, number of source leaves, child octant}

struct HostTransfer {
    std::vector<ot_leaf> from, to;     // both in Morton order
    std::vector<uint64_t> from_keys;   // Morton key of each source leaf's anchor at depth 20
    std::vector<int32_t> table;        // [to.size()][kTransferRow]
    int64_t counts[3] = {0, 0, 0};     // target leaves per kind
};

// Morton key (x least significant) of depth-20 octant coordinates
uint64_t morton_key20(uint32_t x, uint32_t y, uint32_t z);

// Fills everything from the two leaf lists; OT_E_UNSUPPORTED when a target leaf is two or more
// levels finer than the source leaf that contains it.
int make_transfer(const std::vector<ot_leaf>& from, const std::vector<ot_leaf>& to, HostTransfer& out);

struct DeviceTransfer {
    const int32_t* table;
    const ot_leaf* from;
    const uint64_t* from_keys;
    const ot_leaf* to;
    int64_t n_from, n_to;
};

hipError_t launch_transfer(const DeviceTransfer& t, int nvar, const double* from_zipped, double* to_zipped,
                           hipStream_t s);

}  // namespace octfd
