// Drives the library's host sources (csrc/octree_host.cpp, csrc/transfer_host.cpp; no GPU, no HIP call) through
// tree builds, rebuilt leaf lists, regrid plans and the error paths.  tests/test_sanitizers.py builds it with
// g++ -fsanitize=address,undefined -fno-sanitize-recover=all, so that any out-of-bounds access, leak or undefined
// operation ends the run with a report; the expectations below end it with exit code 1.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <random>

#include "octree_host.hpp"
#include "transfer.hpp"

using namespace octfd;

static int failures = 0;
static void expect(bool ok, const char* what)
{
    if (!ok) { std::printf("FAILED: %s\n", what); ++failures; }
}

static uint64_t splitmix(uint64_t& s)
{
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int main(int argc, char** argv)
{
    const int lmax_big = argc > 1 ? std::atoi(argv[1]) : 8;
    // two refinement centres on a circle, at two phases: the trees of a regrid, and the plans both ways
    uint32_t rad[6] = {104857, 87031, 72236, 59956, 49763, 41303};
    HostTree a, b;
    for (int ph = 0; ph < 2; ++ph) {
        const double phi = 1.234 + 0.013 * ph;
        uint32_t pts[6];
        pts[0] = (uint32_t)((0.5 + 0.15 * std::cos(phi)) * 1048576); pts[1] = (uint32_t)((0.5 + 0.15 * std::sin(phi)) * 1048576); pts[2] = 524289;
        pts[3] = (uint32_t)((0.5 - 0.15 * std::cos(phi)) * 1048576); pts[4] = (uint32_t)((0.5 - 0.15 * std::sin(phi)) * 1048576); pts[5] = 524289;
        ot_build_params p{3, (uint32_t)lmax_big, 2, pts, rad, 8, 3, 1};
        expect(build_tree(p, ph ? b : a) == OT_OK, "orbit tree");
        std::printf("orbit tree, phase %d: %zu blocks\n", ph, (ph ? b : a).leaves.size());
    }
    HostTransfer t, t2;
    expect(make_transfer(a.leaves, b.leaves, t) == OT_OK, "plan forwards");
    expect(make_transfer(b.leaves, a.leaves, t2) == OT_OK, "plan backwards");
    expect(t.counts[0] + t.counts[1] + t.counts[2] == (int64_t)b.leaves.size(), "every target leaf has a kind");
    // random trees; the same tree from its shuffled leaf list; a missing and a duplicated leaf
    uint64_t s = 7;
    for (int it = 0; it < 4; ++it) {
        uint32_t pts[6];
        for (auto& v : pts) v = (uint32_t)(splitmix(s) & 0xfffff);
        uint32_t r[3] = {(uint32_t)(20000 + splitmix(s) % 100000), (uint32_t)(20000 + splitmix(s) % 80000), (uint32_t)(splitmix(s) % 60000)};
        ot_build_params p{3, 6, 2, pts, r, 8, 3, 1};
        HostTree h, h2, h3, h4;
        expect(build_tree(p, h) == OT_OK, "random tree");
        std::vector<ot_leaf> lv = h.leaves;
        std::mt19937 g(it);
        std::shuffle(lv.begin(), lv.end(), g);
        expect(tree_from_leaves(lv.data(), lv.size(), h2) == OT_OK, "tree from shuffled leaves");
        expect(h2.ghost == h.ghost && h2.ghost_v == h.ghost_v && h2.vlist == h.vlist && h2.vblk == h.vblk && h2.vneed == h.vneed && h2.units == h.units, "same tables from the leaf list");
        lv.pop_back();
        expect(tree_from_leaves(lv.data(), lv.size(), h3) == OT_E_INCOMPLETE, "missing leaf");
        lv.push_back(lv[0]);
        expect(tree_from_leaves(lv.data(), lv.size(), h4) == OT_E_INCOMPLETE, "duplicate leaf");
    }
    // parameters out of range, including a radius whose square would overflow 64 bits
    {
        uint32_t pts[3] = {1, 2, 3}, r[1] = {5}, huge[1] = {0xffffffffu};
        HostTree h;
        ot_build_params p1{2, 4, 1, pts, r, 8, 3, 1}, p2{3, 20, 1, pts, r, 8, 3, 1}, p3{3, 4, 1, pts, huge, 8, 3, 1}, p4{3, 3, 0, nullptr, nullptr, 8, 3, 1};
        expect(build_tree(p1, h) == OT_E_BADARG, "lmin 2");
        expect(build_tree(p2, h) == OT_E_BADARG, "lmax 20");
        expect(build_tree(p3, h) == OT_E_BADARG, "radius beyond 2^21");
        expect(build_tree(p4, h) == OT_OK && h.leaves.size() == 512, "uniform tree");
    }
    // unbalanced list: level 3 everywhere except one octant refined twice (level 5 next to level 3); and plans
    // across two levels
    {
        std::vector<ot_leaf> lv;
        for (uint32_t z = 0; z < 8; ++z) for (uint32_t y = 0; y < 8; ++y) for (uint32_t x = 0; x < 8; ++x) if (x || y || z) lv.push_back({3, x, y, z});
        for (uint32_t z = 0; z < 4; ++z) for (uint32_t y = 0; y < 4; ++y) for (uint32_t x = 0; x < 4; ++x) lv.push_back({5, x, y, z});
        HostTree h, u3, deep;
        expect(tree_from_leaves(lv.data(), lv.size(), h) == OT_E_UNBALANCED, "unbalanced list");
        ot_build_params p{3, 3, 0, nullptr, nullptr, 8, 3, 1};
        expect(build_tree(p, u3) == OT_OK, "level-3 tree");
        uint32_t pts[3] = {524288, 524288, 524288}, r[2] = {60000, 40000};
        ot_build_params q{3, 5, 1, pts, r, 8, 3, 1};
        expect(build_tree(q, deep) == OT_OK, "three-level tree");
        HostTransfer tt, back;
        expect(make_transfer(u3.leaves, deep.leaves, tt) == OT_E_UNSUPPORTED, "plan across two levels is refused");
        expect(make_transfer(deep.leaves, u3.leaves, back) == OT_OK, "plan that only coarsens");
    }
    std::printf(failures ? "FAILED\n" : "all host checks passed\n");
    return failures ? 1 : 0;
}
