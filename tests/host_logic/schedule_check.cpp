// Host-only check of two derived tables of the library's tree (no GPU, no HIP call): the per-block list of
// coarser sources (corner-only sources last, their count recorded) and the launch schedule of the 24-field
// kernel.  Built with g++ together with csrc/octree_host.cpp by tests/test_library_host.py.
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
    long n_coarse_kind = 0;
    for (long b = 0; b < nb; ++b) {
        const int32_t* row = &t.coarse[b * kCoarseRow];
        // sources named by the ghost table, each exactly once
        int n = 0;
        while (n < 8 && row[2 * n] >= 0) ++n;
        int seen_in_table = 0;
        for (int dir = 0; dir < kDirs; ++dir) {
            const int32_t* e = &t.ghost[(b * kDirs + dir) * kEntry];
            if (e[0] != kCoarser) continue;
            int hit = 0;
            for (int s = 0; s < n; ++s) hit += row[2 * s] == e[1];
            if (hit != 1) return fail("a coarser source of the ghost table is not listed exactly once", b);
            ++seen_in_table;
        }
        if ((n > 0) != (seen_in_table > 0)) return fail("source list and ghost table disagree", b);
        // corner-only sources (ghost part on every axis) come last, and [29] counts the others
        int first_corner = n;
        for (int s = 0; s < n; ++s) {
            const int pk = row[2 * s + 1];
            bool corner = true;
            for (int ax = 0; ax < 3; ++ax) {
                const int lo = (pk >> (4 * ax)) & 3, hi = (pk >> (4 * ax + 2)) & 3;
                if (lo > hi) return fail("empty range", b);
                corner = corner && lo == hi && lo != 1;
            }
            if (corner && first_corner == n) first_corner = s;
            if (!corner && first_corner != n) return fail("a corner-only source precedes another source", b);
        }
        if (row[29] != first_corner) return fail("count of the sources that are not corner-only", b);
        n_coarse_kind += row[29] > 0;
    }
    // schedule: every block once, flag = has such a source; units of kSchedXcds chunks of one kind (one chunk
    // per XCD), padding (-1) only at the end of a kind's last unit
    const size_t unit = static_cast<size_t>(kSchedChunk) * kSchedXcds;
    if (t.sched.size() % unit) return fail("schedule length", -1);
    std::vector<int> times(nb, 0);
    long pad[2] = {0, 0}, count[2] = {0, 0}, units[2] = {0, 0};
    std::vector<int> unit_kind;
    for (size_t c = 0; c < t.sched.size() / unit; ++c) {
        int kind = -1;
        for (size_t i = 0; i < unit; ++i) {
            const int32_t e = t.sched[c * unit + i];
            if (e < 0) continue;
            const int k = (e & kSchedCoarse) ? 1 : 0;
            if (kind >= 0 && k != kind) return fail("a unit mixes the two kinds", e & ~kSchedCoarse);
            kind = k;
        }
        if (kind < 0) return fail("an empty unit", -1);
        unit_kind.push_back(kind);
        ++units[kind];
        for (size_t i = 0; i < unit; ++i) {
            const int32_t e = t.sched[c * unit + i];
            if (e < 0) { ++pad[kind]; continue; }
            if (pad[kind]) return fail("padding before the end of a kind", e & ~kSchedCoarse);
            const long b = e & ~kSchedCoarse;
            if (b >= nb) return fail("block id", b);
            if (((t.coarse[b * kCoarseRow + 29] > 0) ? 1 : 0) != kind) return fail("kind flag", b);
            ++times[b];
            ++count[kind];
        }
    }
    for (long b = 0; b < nb; ++b)
        if (times[b] != 1) return fail("a block is not scheduled exactly once", b);
    if (count[1] != n_coarse_kind || pad[0] >= static_cast<long>(unit) || pad[1] >= static_cast<long>(unit)) return fail("counts", -1);
    // within a kind the blocks keep their (Morton) order
    {
        long last[2] = {-1, -1};
        for (int32_t e : t.sched) {
            if (e < 0) continue;
            const int k = (e & kSchedCoarse) ? 1 : 0;
            const long b = e & ~kSchedCoarse;
            if (b <= last[k]) return fail("order within a kind", b);
            last[k] = b;
        }
    }
    // dealt in proportion: after every unit the two kinds are within one unit of their shares
    long done[2] = {0, 0};
    for (size_t c = 0; c < unit_kind.size(); ++c) {
        ++done[unit_kind[c]];
        if (units[0] && units[1]) {
            const double lag = std::fabs(static_cast<double>(done[0]) / units[0] - static_cast<double>(done[1]) / units[1]);
            if (lag > 1.0 / units[0] + 1.0 / units[1] + 1e-12) return fail("the kinds drift apart in the schedule", static_cast<long>(c));
        }
    }
    const long* chunks = units;
    std::printf("blocks %ld, with a coarser source beyond a corner %ld, units %ld + %ld\n", nb, n_coarse_kind, chunks[0], chunks[1]);
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
