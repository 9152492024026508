// Plan of an inter-grid transfer: one merge walk over the two Morton-ordered leaf lists.  Both
// lists tile the cube, so at every step the current source leaf and the current target leaf
// start at the same position of the space-filling curve and one of them contains the other.
#include "transfer.hpp"

namespace octfd {

uint64_t morton_key20(uint32_t x, uint32_t y, uint32_t z)
{
    uint64_t key = 0;
    for (int b = 0; b < 20; ++b)
        key |= (uint64_t((x >> b) & 1) << (3 * b)) | (uint64_t((y >> b) & 1) << (3 * b + 1)) |
               (uint64_t((z >> b) & 1) << (3 * b + 2));
    return key;
}

namespace {

// is leaf a inside (or equal to) the octant of leaf b
bool inside(const ot_leaf& a, const ot_leaf& b)
{
    if (a.level < b.level) return false;
    const uint32_t sh = a.level - b.level;
    return (a.ix >> sh) == b.ix && (a.iy >> sh) == b.iy && (a.iz >> sh) == b.iz;
}

}  // namespace

int make_transfer(const std::vector<ot_leaf>& from, const std::vector<ot_leaf>& to, HostTransfer& out)
{
    const size_t nf = from.size(), nt = to.size();
    if (nf == 0 || nt == 0 || nf >= (size_t(1) << 31) || nt >= (size_t(1) << 31)) return OT_E_BADARG;
    out.from = from;
    out.to = to;
    out.from_keys.resize(nf);
    for (size_t i = 0; i < nf; ++i) {
        const uint32_t sh = 20 - from[i].level;
        out.from_keys[i] = morton_key20(from[i].ix << sh, from[i].iy << sh, from[i].iz << sh);
    }
    out.table.assign(nt * kTransferRow, 0);
    out.counts[0] = out.counts[1] = out.counts[2] = 0;
    auto row = [&](size_t j, int32_t kind, size_t first, size_t count, int32_t octant) {
        int32_t* r = &out.table[j * kTransferRow];
        r[0] = kind; r[1] = static_cast<int32_t>(first); r[2] = static_cast<int32_t>(count); r[3] = octant;
        ++out.counts[kind];
    };
    size_t i = 0, j = 0;
    while (j < nt) {
        if (i >= nf) return OT_E_INCOMPLETE;
        const ot_leaf F = from[i], T = to[j];
        if (F.level == T.level) {
            if (!inside(F, T)) return OT_E_INCOMPLETE;
            row(j, kCopy, i, 1, 0);
            ++i; ++j;
        } else if (F.level < T.level) {            // source coarser: all its target descendants, one level down
            if (!inside(T, F)) return OT_E_INCOMPLETE;
            while (j < nt && inside(to[j], F)) {
                if (to[j].level != F.level + 1) return OT_E_UNSUPPORTED;
                row(j, kProlong, i, 1, static_cast<int32_t>((to[j].ix & 1) | ((to[j].iy & 1) << 1) | ((to[j].iz & 1) << 2)));
                ++j;
            }
            ++i;
        } else {                                   // source finer: the run of source leaves inside the target leaf
            if (!inside(F, T)) return OT_E_INCOMPLETE;
            const size_t first = i;
            while (i < nf && inside(from[i], T)) ++i;
            row(j, kInject, first, i - first, 0);
            ++j;
        }
    }
    return i == nf ? OT_OK : OT_E_INCOMPLETE;
}

}  // namespace octfd
