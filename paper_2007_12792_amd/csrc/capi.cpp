// C ABI of liboctfd (see include/octfd.h): argument checking, tree ownership, lazy upload of the
// index tables, and the sequencing of kernel launches.  No arithmetic of the method lives here.
#include <hip/hip_runtime.h>

#include <atomic>
#include <new>

#include "kernels.hpp"
#include "octfd.h"
#include "octree_host.hpp"
#include "transfer.hpp"

using namespace octfd;

// The device copies of the tables are a cache inside the opaque handle: the device entry points take the tree
// as const and fill the cache on first use (octree_upload fills it ahead of time).
struct ot_tree {
    HostTree host;
    mutable char* d_base = nullptr;    // one allocation for all tables
    mutable DeviceTree dev{};          // views into it
    mutable int device = -1;           // device the tables live on, -1 = not uploaded
    // virtual blocks of the input of rhs_eval_zipped, which has no workspace argument: allocated by its first
    // call that needs them (a tree with level jumps), kept until octree_free
    mutable double* d_virt = nullptr;
    mutable size_t virt_bytes = 0;
};

struct ot_transfer {
    HostTransfer host;
    char* d_base = nullptr;   // one allocation: table, source leaves, source keys, target leaves
    DeviceTransfer dev{};
    int device = -1;
};

// Workspace of rk_step_static: one copy per GPU, held by the code object until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels receive the resolved address (g_static_ws).
static __device__ __align__(256) unsigned char scratch[OT_STATIC_WORKSPACE_BYTES];

namespace {

std::atomic<int> g_last_hip{0};

int hip_fail(hipError_t e);

constexpr int kMaxDevices = 64;
std::atomic<void*> g_static_ws[kMaxDevices];   // per device: address of `scratch` there, null until resolved

// once per device, with that device current (called from the upload of a tree's tables)
int resolve_static_workspace(int dev)
{
    if (dev < 0 || dev >= kMaxDevices) return OT_E_UNSUPPORTED;
    if (g_static_ws[dev].load()) return OT_OK;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256) return OT_E_HIP;
    g_static_ws[dev].store(ptr);
    return OT_OK;
}

int hip_fail(hipError_t e)
{
    g_last_hip.store(static_cast<int>(e));
    return (e == hipErrorNoDevice || e == hipErrorInvalidDevice || e == hipErrorInsufficientDriver) ? OT_E_NODEVICE
           : (e == hipErrorOutOfMemory)                                                             ? OT_E_NOMEM
                                                                                                    : OT_E_HIP;
}

// the tables live on the device that was current at the first device call; later calls must run there
int same_device(int device)
{
    int cur = -1;
    const hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return hip_fail(e);
    return cur == device ? OT_OK : OT_E_UNSUPPORTED;
}

int ensure_device(const ot_tree* t)
{
    if (t->device >= 0) return same_device(t->device);
    // kernels address one variable's zipped array with 32-bit byte offsets
    if (t->host.leaves.size() >= (size_t(1) << 20)) return OT_E_UNSUPPORTED;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess) return hip_fail(e);
    if (ndev <= 0) return OT_E_NODEVICE;
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return hip_fail(e);
    // one allocation for all tables, each part 256-byte aligned
    const HostTree& h = t->host;
    constexpr int kParts = 6;
    auto ibytes = [](const std::vector<int32_t>& v) { return v.size() * sizeof(int32_t); };
    const void* part[kParts] = {h.leaves.data(), h.ghost_v.data(), h.vblk.data(), h.vlist.data(), h.units.data(), h.vneed.data()};
    const size_t bytes[kParts] = {h.leaves.size() * sizeof(ot_leaf), ibytes(h.ghost_v), ibytes(h.vblk), ibytes(h.vlist), ibytes(h.units), ibytes(h.vneed)};
    size_t off[kParts + 1] = {0};
    for (int i = 0; i < kParts; ++i) off[i + 1] = off[i] + (bytes[i] + 255) / 256 * 256;
    char* base = nullptr;
    if ((e = hipMalloc(reinterpret_cast<void**>(&base), off[kParts])) != hipSuccess) return hip_fail(e);
    for (int i = 0; i < kParts && e == hipSuccess; ++i)
        if (bytes[i]) e = hipMemcpy(base + off[i], part[i], bytes[i], hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(base);
        return hip_fail(e);
    }
    auto ints = [&](int i) { return reinterpret_cast<const int32_t*>(base + off[i]); };
    t->d_base = base;
    t->dev = DeviceTree{reinterpret_cast<const ot_leaf*>(base + off[0]), static_cast<int64_t>(h.leaves.size()),
                        ints(1), ints(2), ints(3), h.n_virt, ints(4), static_cast<int64_t>(h.units.size()), ints(5)};
    t->device = dev;
    return resolve_static_workspace(dev);
}

int ensure_device(ot_transfer* p)
{
    if (p->device >= 0) return same_device(p->device);
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess) return hip_fail(e);
    if (ndev <= 0) return OT_E_NODEVICE;
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return hip_fail(e);
    const HostTransfer& h = p->host;
    auto up = [](size_t n) { return (n + 255) / 256 * 256; };
    const size_t nt = h.table.size() * sizeof(int32_t), nf = h.from.size() * sizeof(ot_leaf);
    const size_t nk = h.from_keys.size() * sizeof(uint64_t), no = h.to.size() * sizeof(ot_leaf);
    const size_t of = up(nt), ok = of + up(nf), oo = ok + up(nk);
    char* base = nullptr;
    if ((e = hipMalloc(reinterpret_cast<void**>(&base), oo + no)) != hipSuccess) return hip_fail(e);
    e = hipMemcpy(base, h.table.data(), nt, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(base + of, h.from.data(), nf, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(base + ok, h.from_keys.data(), nk, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(base + oo, h.to.data(), no, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(base);
        return hip_fail(e);
    }
    p->d_base = base;
    p->dev = DeviceTransfer{reinterpret_cast<const int32_t*>(base), reinterpret_cast<const ot_leaf*>(base + of),
                            reinterpret_cast<const uint64_t*>(base + ok), reinterpret_cast<const ot_leaf*>(base + oo),
                            static_cast<int64_t>(h.from.size()), static_cast<int64_t>(h.to.size())};
    p->device = dev;
    return OT_OK;
}

DeviceTree dev_view(const ot_tree* t) { return t->dev; }

bool kind_ok(int k) { return k >= OT_RHS_DERIVS && k <= OT_RHS_SYN24; }

// the tree's own array of virtual blocks, for the calls that have no workspace argument: at least `bytes` large
int ensure_virtual_scratch(const ot_tree* tree, size_t bytes)
{
    if (bytes <= tree->virt_bytes) return OT_OK;
    hipError_t e = hipSuccess;
    if (tree->d_virt) e = hipFree(tree->d_virt);   // synchronises with earlier work on the old array
    tree->d_virt = nullptr;
    tree->virt_bytes = 0;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&tree->d_virt), bytes);
    if (e != hipSuccess) return hip_fail(e);
    tree->virt_bytes = bytes;
    return OT_OK;
}

// bytes of the virtual blocks of one input vector of a kind
size_t virtual_bytes(const ot_tree* t, int kind)
{
    return static_cast<size_t>(ot_rhs_nvar_in(static_cast<ot_rhs_kind>(kind))) * static_cast<size_t>(t->host.n_virt) * 512 * sizeof(double);
}

// data arrays hold doubles: anything else cannot be a valid array and would fault in the kernels
bool aligned8(const void* p) { return reinterpret_cast<uintptr_t>(p) % 8 == 0; }

}  // namespace

extern "C" {

int octree_build(const ot_build_params* params, ot_tree** out)
{
    if (!params || !out) return OT_E_BADARG;
    *out = nullptr;
    ot_tree* t = new (std::nothrow) ot_tree;
    if (!t) return OT_E_NOMEM;
    int rc;
    try { rc = build_tree(*params, t->host); } catch (const std::bad_alloc&) { rc = OT_E_NOMEM; }
    if (rc != OT_OK) { delete t; return rc; }
    *out = t;
    return OT_OK;
}

int octree_from_leaves(const ot_leaf* leaves, size_t n, uint32_t pad, ot_tree** out)
{
    if (!leaves || !out || n == 0) return OT_E_BADARG;
    *out = nullptr;
    if (pad != 3) return OT_E_UNSUPPORTED;
    ot_tree* t = new (std::nothrow) ot_tree;
    if (!t) return OT_E_NOMEM;
    int rc;
    try { rc = tree_from_leaves(leaves, n, t->host); } catch (const std::bad_alloc&) { rc = OT_E_NOMEM; }
    if (rc != OT_OK) { delete t; return rc; }
    *out = t;
    return OT_OK;
}

int octree_num_blocks(const ot_tree* tree, int64_t* nb)
{
    if (!tree || !nb) return OT_E_BADARG;
    *nb = static_cast<int64_t>(tree->host.leaves.size());
    return OT_OK;
}

int octree_get_leaves(const ot_tree* tree, ot_leaf* out, size_t cap)
{
    if (!tree || !out || cap < tree->host.leaves.size()) return OT_E_BADARG;
    for (size_t i = 0; i < tree->host.leaves.size(); ++i) out[i] = tree->host.leaves[i];
    return OT_OK;
}

int octree_get_ghost_table(const ot_tree* tree, int32_t* out, size_t cap)
{
    if (!tree || !out || cap < tree->host.ghost.size()) return OT_E_BADARG;
    for (size_t i = 0; i < tree->host.ghost.size(); ++i) out[i] = tree->host.ghost[i];
    return OT_OK;
}

int octree_upload(ot_tree* tree)
{
    if (!tree) return OT_E_BADARG;
    return ensure_device(tree);
}

int octree_free(ot_tree* tree)
{
    if (!tree) return OT_OK;
    int rc = OT_OK;
    if (tree->device >= 0) {
        hipError_t e = hipFree(tree->d_base);
        if (e != hipSuccess) rc = hip_fail(e);
        if (tree->d_virt && (e = hipFree(tree->d_virt)) != hipSuccess) rc = hip_fail(e);
    }
    delete tree;
    return rc;
}

int ot_rhs_nvar_in(ot_rhs_kind kind)
{
    switch (kind) {
    case OT_RHS_DERIVS: return 1;
    case OT_RHS_WAVE: return 2;
    case OT_RHS_BURGERS: return 1;
    case OT_RHS_SYN24: return 24;
    default: return OT_E_BADARG;
    }
}

int ot_rhs_nvar_out(ot_rhs_kind kind)
{
    switch (kind) {
    case OT_RHS_DERIVS: return 4;
    case OT_RHS_WAVE: return 2;
    case OT_RHS_BURGERS: return 1;
    case OT_RHS_SYN24: return 24;
    default: return OT_E_BADARG;
    }
}

// both ghost rules: fill the virtual blocks of the input (that is where the rules differ), then gather
static int unzip_any(const ot_tree* tree, bool centred, int nvar, const double* zipped_dev, double* padded_dev, void* hip_stream)
{
    if (!tree || nvar <= 0 || !zipped_dev || !padded_dev || !aligned8(zipped_dev) || !aligned8(padded_dev)) return OT_E_BADARG;
    if (int rc = ensure_device(tree)) return rc;   // < 2^20 blocks, and the grid is at most 8 workgroups per block
    const size_t vbytes = static_cast<size_t>(nvar) * static_cast<size_t>(tree->host.n_virt) * 512 * sizeof(double);
    if (int rc = ensure_virtual_scratch(tree, vbytes)) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const DeviceTree dv = dev_view(tree);
    hipError_t e = centred ? launch_virtual_centred(dv, tree->host.vlevel_start, nvar, zipped_dev, tree->d_virt, s)
                           : launch_virtual(dv, nvar, zipped_dev, tree->d_virt, s);
    if (e == hipSuccess) e = launch_unzip(dv, nvar, zipped_dev, tree->d_virt, padded_dev, s);
    return e == hipSuccess ? OT_OK : hip_fail(e);
}

int unzip(const ot_tree* tree, int nvar, const double* zipped_dev, double* padded_dev, void* hip_stream)
{
    return unzip_any(tree, false, nvar, zipped_dev, padded_dev, hip_stream);
}

int unzip_centred(const ot_tree* tree, int nvar, const double* zipped_dev, double* padded_dev, void* hip_stream)
{
    return unzip_any(tree, true, nvar, zipped_dev, padded_dev, hip_stream);
}

int zip(const ot_tree* tree, int nvar, const double* padded_dev, double* zipped_dev, void* hip_stream)
{
    if (!tree || nvar <= 0 || !zipped_dev || !padded_dev || !aligned8(zipped_dev) || !aligned8(padded_dev)) return OT_E_BADARG;
    if (tree->host.leaves.size() * static_cast<size_t>(nvar) > 0x7fffffffu) return OT_E_UNSUPPORTED;   // one workgroup each
    if (int rc = ensure_device(tree)) return rc;
    hipError_t e = launch_zip(dev_view(tree), nvar, padded_dev, zipped_dev, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OT_OK : hip_fail(e);
}

int rhs_eval(const ot_tree* tree, ot_rhs_kind kind, const ot_rhs_params* params, const double* padded_dev,
             double* rhs_padded_dev, void* hip_stream)
{
    if (!tree || !kind_ok(kind) || !params || !padded_dev || !rhs_padded_dev || !aligned8(padded_dev) || !aligned8(rhs_padded_dev))
        return OT_E_BADARG;
    if (int rc = ensure_device(tree)) return rc;
    RhsArgs a{padded_dev, rhs_padded_dev, nullptr, nullptr, nullptr, rhs_padded_dev, 0.0, params->ko_sigma};
    hipError_t e = launch_rhs(dev_view(tree), kind, false, kOutPadded, a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OT_OK : hip_fail(e);
}

int rhs_eval_zipped(const ot_tree* tree, ot_rhs_kind kind, const ot_rhs_params* params, const double* zipped_dev,
                    double* rhs_zipped_dev, void* hip_stream)
{
    if (!tree || !kind_ok(kind) || !params || !zipped_dev || !rhs_zipped_dev || !aligned8(zipped_dev) || !aligned8(rhs_zipped_dev))
        return OT_E_BADARG;
    if (int rc = ensure_device(tree)) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const DeviceTree dv = dev_view(tree);
    const size_t vbytes = virtual_bytes(tree, kind);
    if (int rc = ensure_virtual_scratch(tree, vbytes)) return rc;
    if (vbytes) {
        hipError_t e = launch_virtual(dv, ot_rhs_nvar_in(kind), zipped_dev, tree->d_virt, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    RhsArgs a{zipped_dev, rhs_zipped_dev, nullptr, nullptr, vbytes ? tree->d_virt : nullptr, rhs_zipped_dev, 0.0, params->ko_sigma};
    hipError_t e = launch_rhs(dv, kind, true, kOutZipped, a, s);
    return e == hipSuccess ? OT_OK : hip_fail(e);
}

int rk_workspace_bytes(const ot_tree* tree, ot_rhs_kind kind, size_t* bytes)
{
    if (!tree || !kind_ok(kind) || !bytes) return OT_E_BADARG;
    if (ot_rhs_nvar_in(kind) != ot_rhs_nvar_out(kind)) return OT_E_UNSUPPORTED;
    // three zipped vectors, then the virtual blocks of the current stage vector
    *bytes = 3 * static_cast<size_t>(ot_rhs_nvar_in(kind)) * tree->host.leaves.size() * 512 * sizeof(double) + virtual_bytes(tree, kind);
    return OT_OK;
}

// checks shared by the stepping calls: u holds doubles, the workspace is large enough and 256-byte aligned, and the
// two do not overlap (the stage kernels read ghosts of u while they write stage vectors into the workspace)
static int check_step_buffers(const double* u, size_t u_bytes, const void* ws, size_t ws_bytes, size_t need)
{
    if (ws_bytes < need) return OT_E_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % 256 || !aligned8(u)) return OT_E_BADARG;
    const uintptr_t u0 = reinterpret_cast<uintptr_t>(u), w0 = reinterpret_cast<uintptr_t>(ws);
    if (u0 < w0 + need && w0 < u0 + u_bytes) return OT_E_BADARG;
    return OT_OK;
}

// the four stage launches of rk_step on tables that are already on the device
static int rk_step_launch(const ot_tree* tree, ot_rhs_kind kind, const ot_rhs_params* params, double dt, double* u,
                          void* workspace_dev, size_t need, hipStream_t s, bool centred = false)
{
    const size_t vbytes = virtual_bytes(tree, kind);
    const size_t len = (need - vbytes) / (3 * sizeof(double));
    double* acc = static_cast<double*>(workspace_dev);
    double* sa = acc + len;
    double* sb = sa + len;
    double* virt = vbytes ? sb + len : nullptr;
    const DeviceTree dv = dev_view(tree);
    const double sg = params->ko_sigma;
    // stage vectors ping-pong between sa and sb: a stage reads ghosts of the vector it was given
    // while writing the next one, so the two must be different arrays
    const RhsArgs st[4] = {
        {u, sa, acc, u, virt, sa, 0.5 * dt, sg},    // k1 = F(u):   acc = k1,        sa = u + dt/2 k1
        {sa, sb, acc, u, virt, sb, 0.5 * dt, sg},   // k2 = F(sa):  acc += 2 k2,     sb = u + dt/2 k2
        {sb, sa, acc, u, virt, sa, dt, sg},         // k3 = F(sb):  acc += 2 k3,     sa = u + dt k3
        {sa, nullptr, acc, u, virt, sb, dt / 6.0, sg}};   // k4 = F(sa):  u += dt/6 (acc + k4); sb is free scratch
    const Epilogue ep[4] = {kRkFirst, kRkMiddle, kRkMiddle, kRkLast};
    for (int i = 0; i < 4; ++i) {
        // the virtual blocks of this stage's input first; the stream orders them before the stage kernel and
        // after the previous stage's reads of the same array
        hipError_t e = hipSuccess;
        if (vbytes && centred) e = launch_virtual_centred(dv, tree->host.vlevel_start, ot_rhs_nvar_in(kind), st[i].in, virt, s);
        else if (vbytes) e = launch_virtual(dv, ot_rhs_nvar_in(kind), st[i].in, virt, s);
        if (e == hipSuccess) e = launch_rhs(dv, kind, true, ep[i], st[i], s);
        if (e != hipSuccess) return hip_fail(e);
    }
    return OT_OK;
}

int rk_step(const ot_tree* tree, ot_rhs_kind kind, const ot_rhs_params* params, double dt, double* u_zipped_dev,
            void* workspace_dev, size_t workspace_bytes, void* hip_stream)
{
    if (!tree || !kind_ok(kind) || !params || !u_zipped_dev || !workspace_dev) return OT_E_BADARG;
    size_t need = 0;
    if (int rc = rk_workspace_bytes(tree, kind, &need)) return rc;
    if (int rc = check_step_buffers(u_zipped_dev, (need - virtual_bytes(tree, kind)) / 3, workspace_dev, workspace_bytes, need)) return rc;
    if (int rc = ensure_device(tree)) return rc;
    return rk_step_launch(tree, kind, params, dt, u_zipped_dev, workspace_dev, need, static_cast<hipStream_t>(hip_stream));
}

int rk_step_static(const ot_tree* tree, ot_rhs_kind kind, const ot_rhs_params* params, double dt, double* u_zipped_dev,
                   void* hip_stream)
{
    if (!tree || !kind_ok(kind) || !params || !u_zipped_dev) return OT_E_BADARG;
    size_t need = 0;
    if (int rc = rk_workspace_bytes(tree, kind, &need)) return rc;
    if (need > OT_STATIC_WORKSPACE_BYTES) return OT_E_WORKSPACE;
    // no upload here (it allocates): the tables and the array's address must be in place already
    if (tree->device < 0 || tree->device >= kMaxDevices) return OT_E_UNSUPPORTED;
    if (int rc = same_device(tree->device)) return rc;
    void* ws = g_static_ws[tree->device].load();
    if (!ws) return OT_E_UNSUPPORTED;
    if (int rc = check_step_buffers(u_zipped_dev, (need - virtual_bytes(tree, kind)) / 3, ws, OT_STATIC_WORKSPACE_BYTES, need)) return rc;
    return rk_step_launch(tree, kind, params, dt, u_zipped_dev, ws, need, static_cast<hipStream_t>(hip_stream));
}

int rk_centred_workspace_bytes(const ot_tree* tree, ot_rhs_kind kind, size_t* bytes)
{
    return rk_workspace_bytes(tree, kind, bytes);   // the two ghost rules fill the same virtual blocks
}

int rk_step_centred(const ot_tree* tree, ot_rhs_kind kind, const ot_rhs_params* params, double dt, double* u_zipped_dev,
                    void* workspace_dev, size_t workspace_bytes, void* hip_stream)
{
    if (!tree || !kind_ok(kind) || !params || !u_zipped_dev || !workspace_dev) return OT_E_BADARG;
    size_t need = 0;
    if (int rc = rk_workspace_bytes(tree, kind, &need)) return rc;
    if (int rc = check_step_buffers(u_zipped_dev, (need - virtual_bytes(tree, kind)) / 3, workspace_dev, workspace_bytes, need)) return rc;
    if (int rc = ensure_device(tree)) return rc;
    return rk_step_launch(tree, kind, params, dt, u_zipped_dev, workspace_dev, need, static_cast<hipStream_t>(hip_stream), true);
}

int regrid_plan(const ot_tree* from, const ot_tree* to, ot_transfer** out)
{
    if (!from || !to || !out) return OT_E_BADARG;
    *out = nullptr;
    ot_transfer* p = new (std::nothrow) ot_transfer;
    if (!p) return OT_E_NOMEM;
    int rc;
    try { rc = make_transfer(from->host.leaves, to->host.leaves, p->host); } catch (const std::bad_alloc&) { rc = OT_E_NOMEM; }
    if (rc != OT_OK) { delete p; return rc; }
    *out = p;
    return OT_OK;
}

int regrid_table(const ot_transfer* plan, int32_t* out, size_t cap)
{
    if (!plan || !out || cap < plan->host.table.size()) return OT_E_BADARG;
    for (size_t i = 0; i < plan->host.table.size(); ++i) out[i] = plan->host.table[i];
    return OT_OK;
}

int regrid_transfer(ot_transfer* plan, int nvar, const double* from_zipped_dev, double* to_zipped_dev, void* hip_stream)
{
    if (!plan || nvar <= 0 || !from_zipped_dev || !to_zipped_dev) return OT_E_BADARG;
    if (int rc = ensure_device(plan)) return rc;
    hipError_t e = launch_transfer(plan->dev, nvar, from_zipped_dev, to_zipped_dev, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OT_OK : hip_fail(e);
}

int regrid_free(ot_transfer* plan)
{
    if (!plan) return OT_OK;
    int rc = OT_OK;
    if (plan->device >= 0) {
        hipError_t e = hipFree(plan->d_base);
        if (e != hipSuccess) rc = hip_fail(e);
    }
    delete plan;
    return rc;
}

const char* ot_strerror(int status)
{
    switch (status) {
    case OT_OK: return "ok";
    case OT_E_BADARG: return "bad argument";
    case OT_E_NOMEM: return "out of memory";
    case OT_E_UNBALANCED: return "leaves are not 2:1 balanced over the 26 neighbours";
    case OT_E_INCOMPLETE: return "leaves do not tile the cube exactly once";
    case OT_E_WORKSPACE: return "workspace too small";
    case OT_E_HIP: return "HIP call failed";
    case OT_E_NODEVICE: return "no usable GPU";
    case OT_E_UNSUPPORTED: return "unsupported parameter";
    default: return "unknown status";
    }
}

int ot_last_hip_error(void) { return g_last_hip.load(); }

}  // extern "C"
