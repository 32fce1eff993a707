// Memory-safety fuzz of the decode plan builder (host code only; built with the address and undefined-behaviour
// sanitizers by tests/test_library_host.py).  Random forests with the sharing structure forks produce - a
// thread's table is its root path's blocks, refcounts count the live holders, internal nodes end on block
// boundaries - are planned under random geometry and policy parameters; the plan is checked for coverage:
// every row group of every listed thread must be shown exactly the blocks of its thread's table, once, and
// every index in the plan must lie inside its array (the sanitizers watch the builder's own accesses).
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "plan.hpp"

using namespace apar;

#define CHECK(c)                                                                   \
    do {                                                                           \
        if (!(c)) {                                                                \
            std::fprintf(stderr, "seed %d: check failed: %s (line %d)\n", seed, #c, __LINE__); \
            return 1;                                                              \
        }                                                                          \
    } while (0)

static int one(int seed) {
    std::mt19937 rng(seed);
    auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
    // forest: node = (parent, own blocks); leaves are the threads
    struct Node { int parent; std::vector<int32_t> blocks; int last_valid; std::vector<int> kids; };
    std::vector<Node> nodes;
    int32_t next_block = 0;
    const int n_roots = rnd(1, 3), max_nodes = rnd(4, 400);
    for (int r = 0; r < n_roots; ++r) nodes.push_back(Node{-1, {}, 16, {}});
    while ((int)nodes.size() < max_nodes) {
        const int p = rnd(0, (int)nodes.size() - 1);
        const int fan = rnd(1, rng() % 8 == 0 ? 200 : 6);
        for (int k = 0; k < fan; ++k) {
            nodes[p].kids.push_back((int)nodes.size());
            nodes.push_back(Node{p, {}, 16, {}});
        }
    }
    for (Node& nd : nodes) {
        const bool leaf = nd.kids.empty();
        const int nb = leaf ? rnd(0, 6) : rnd(1, rng() % 6 == 0 ? 300 : 5);  // a leaf may have no block of its own
        for (int b = 0; b < nb; ++b) nd.blocks.push_back(next_block++);
        nd.last_valid = (leaf && nb > 0) ? rnd(1, 16) : 16;
    }
    // a leaf without blocks of its own under a parent: it ends at the parent's segment.  Roots that are leaves need a block.
    for (Node& nd : nodes)
        if (nd.parent < 0 && nd.kids.empty() && nd.blocks.empty()) nd.blocks.push_back(next_block++);
    // a node all of whose children end at it (threads listed right after their fork) may end on an open block
    for (Node& nd : nodes) {
        if (nd.kids.empty()) continue;
        bool all_end_here = true;
        for (int k : nd.kids) all_end_here = all_end_here && nodes[k].kids.empty() && nodes[k].blocks.empty();
        if (all_end_here) nd.last_valid = rnd(1, 16);
    }
    std::vector<int32_t> refcount(next_block + 8, 0);
    std::vector<std::vector<int32_t>> tables;
    std::vector<int64_t> lens;
    for (size_t i = 0; i < nodes.size(); ++i) {
        if (!nodes[i].kids.empty()) continue;
        std::vector<int> path;
        for (int a = (int)i; a >= 0; a = nodes[a].parent) path.push_back(a);
        std::vector<int32_t> t;
        for (auto it = path.rbegin(); it != path.rend(); ++it) t.insert(t.end(), nodes[*it].blocks.begin(), nodes[*it].blocks.end());
        for (int32_t b : t) refcount[b] += 1;
        const int lv = nodes[i].blocks.empty() ? nodes[nodes[i].parent].last_valid : nodes[i].last_valid;
        tables.push_back(t);
        lens.push_back((int64_t)(t.size() - 1) * 16 + lv);
    }
    const int n = (int)tables.size();
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::shuffle(order.begin(), order.end(), rng);
    std::vector<PlanThreadView> views(n);
    for (int i = 0; i < n; ++i) views[i] = PlanThreadView{tables[order[i]].data(), (int32_t)tables[order[i]].size(), lens[order[i]]};
    std::vector<int32_t> seg_of(refcount.size(), -1);
    PlanHost ph;
    for (int round = 0; round < 3; ++round) {
        PlanParams prm{};
        const int rpts[] = {1, 2, 4, 5, 8, 16, 20, 40, 64};
        prm.rows_per_thread = rpts[rng() % 9];
        const int caps[] = {1, 2, 5, 16, 64, 512};
        prm.max_unit_tiles = caps[rng() % 6];
        prm.allow_direct = rng() % 8 != 0;
        prm.fuse = rng() % 8 != 0;
        prm.inline_shared = rng() % 2;
        const int mrows[] = {0, 1, 64, 256};
        prm.matrix_min_rows = mrows[rng() % 4];
        const int mblk[] = {1, 3, 128};
        prm.matrix_min_blocks = mblk[rng() % 3];
        CHECK(build_plan(views.data(), n, refcount.data(), seg_of.data(), prm, ph) == 0);
        for (int32_t x : seg_of) CHECK(x == -1);
        const int n_sl = (prm.rows_per_thread + 15) / 16;
        // coverage: row group -> multiset of (block, valid)
        std::vector<std::map<int32_t, int>> seen((size_t)n * n_sl);
        const size_t n_tiles = ph.tiles.size();
        auto show = [&](const TileRef& t, int base, int g, int& err) {
            const int lo = t.meta & 1023, hi = (t.meta >> 10) & 1023, valid = (t.meta >> 20) & 31;
            if (valid < 1 || valid > 16 || lo >= hi) err = 1;
            if (g - base >= lo && g - base < hi) seen[g][t.blk] += valid;
        };
        for (const WgDesc& wg : ph.wgs) {
            CHECK(wg.coop_ofs >= 0 && wg.n_coop >= 0 && (size_t)wg.coop_ofs + wg.n_coop <= n_tiles);
            for (int k = 0; k < 4; ++k) {
                const WaveItem& wi = wg.w[k];
                CHECK(wi.n_grp >= 0 && wi.n_tiles >= 0);
                if (wi.n_grp == 0) continue;
                CHECK(wi.tile_ofs >= 0 && (size_t)wi.tile_ofs + wi.n_tiles <= n_tiles);
                CHECK(wi.grp_lo >= 0 && wi.grp_lo + wi.n_grp <= n * n_sl);
                int err = 0;
                for (int g = wi.grp_lo; g < wi.grp_lo + wi.n_grp; ++g) {
                    for (int t = 0; t < wg.n_coop; ++t) show(ph.tiles[wg.coop_ofs + t], wg.grp_base, g, err);
                    for (int t = 0; t < wi.n_tiles; ++t) show(ph.tiles[wi.tile_ofs + t], wi.grp_lo, g, err);
                }
                CHECK(!err);
            }
        }
        CHECK((int)ph.dfs_threads.size() == n);
        for (int rank = 0; rank < n; ++rank) {
            const int i = ph.dfs_threads[rank];
            CHECK(i >= 0 && i < n);
            const std::vector<int32_t>& tb = tables[order[i]];
            const int64_t len = lens[order[i]];
            for (int sl = 0; sl < n_sl; ++sl) {
                const std::map<int32_t, int>& got = seen[(size_t)rank * n_sl + sl];
                CHECK(got.size() == tb.size());
                int64_t total = 0;
                for (int32_t b : tb) {
                    auto it = got.find(b);
                    CHECK(it != got.end() && it->second <= 16);
                    total += it->second;
                }
                CHECK(total == len);
            }
            CHECK(ph.path_ofs[i] <= ph.path_ofs[i + 1] && (size_t)ph.path_ofs[i + 1] <= ph.path_ids.size());
            for (int p = ph.path_ofs[i]; p < ph.path_ofs[i + 1]; ++p) CHECK(ph.path_ids[p] >= 0 && ph.path_ids[p] < ph.n_partial_rows);
        }
    }
    return 0;
}

int main(int argc, char** argv) {
    const int first = argc > 1 ? std::atoi(argv[1]) : 0, count = argc > 2 ? std::atoi(argv[2]) : 200;
    for (int seed = first; seed < first + count; ++seed)
        if (one(seed)) return 1;
    std::printf("ok: %d forests\n", count);
    return 0;
}
