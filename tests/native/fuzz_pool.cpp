// Memory-safety fuzz of the library's host side on bookkeeping-only pools (no GPU): allocator, copy-on-write,
// batched appends, candidate commits, plans, the Algorithm 1 controller and the serving loop, driven by random
// operation sequences on pools small enough to run out of blocks.  Built by tests/test_library_host.py as
// plain host C++ with the address and undefined-behaviour sanitizers; the kernels' launchers are stubs (a
// bookkeeping-only pool never calls them).  Checks: statuses are the documented ones, a failed call leaves the
// counters as they were, used + free blocks = pool size, refcounts equal the number of live holders.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "apar_internal.hpp"

namespace apar {
hipError_t fixed_workspace_of_device(int, char** out) { static char nothing[256]; *out = nothing; return hipSuccess; }
hipError_t launch_append_rows(const Shape&, void*, const void*, const void*, const int32_t*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_block_copies(const Shape&, void*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_seal_blocks(const Shape&, void*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_read_rows(const Shape&, const void*, const int32_t*, int, void*, void*, hipStream_t) { std::abort(); }
hipError_t launch_scatter_words(int32_t*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_attention_partial(const Shape&, const void*, const void*, const PlanDev&, int, PartialBuf, const void*, const void*,
                                    const uint8_t*, void*, ClassStreams&, hipStream_t) { std::abort(); }
hipError_t launch_prefill_bf16(const Shape&, const void*, const void*, const PrefillWg*, const int32_t*, int, void*, hipStream_t) { std::abort(); }
hipError_t launch_attention_units_bf16(const Shape&, const void*, const void*, const PlanDev&, int, int, int, PartialBuf, hipStream_t) { std::abort(); }
hipError_t launch_merge(const Shape&, const PlanDev&, PartialBuf, const void*, const void*, const void*, const uint8_t*, int, void*,
                        hipStream_t) { std::abort(); }
}  // namespace apar

#define CHECK(c)                                                                                  \
    do {                                                                                          \
        if (!(c)) {                                                                               \
            std::fprintf(stderr, "seed %d: check failed: %s (line %d)\n", seed, #c, __LINE__);    \
            return 1;                                                                             \
        }                                                                                         \
    } while (0)

// The plan of the last decode call must read, for every row group of every listed thread, exactly the blocks of
// the thread's table, each once, with fill counts that add up to its length; every list holds its full tiles first.
static int plan_covers_tables(apar_pool* p, const std::vector<apar_thread>& ids, int seed) {
    int64_t n_wgs = 0, n_tiles = 0, n_dfs = 0, n_geom = 0;
    apar_last_plan_export(p, APAR_PLAN_WORKGROUPS, nullptr, 0, &n_wgs);  // (refused for its size: only the count comes back)
    apar_last_plan_export(p, APAR_PLAN_TILES, nullptr, 0, &n_tiles);
    std::vector<int32_t> wgs(n_wgs + 1), tiles(n_tiles + 1), dfs(ids.size() + 1), geom(3);
    CHECK(apar_last_plan_export(p, APAR_PLAN_WORKGROUPS, wgs.data(), (int64_t)wgs.size(), &n_wgs) == APAR_OK);
    CHECK(apar_last_plan_export(p, APAR_PLAN_TILES, tiles.data(), (int64_t)tiles.size(), &n_tiles) == APAR_OK);
    CHECK(apar_last_plan_export(p, APAR_PLAN_DFS_THREADS, dfs.data(), (int64_t)dfs.size(), &n_dfs) == APAR_OK);
    CHECK(apar_last_plan_export(p, APAR_PLAN_GEOMETRY, geom.data(), 3, &n_geom) == APAR_OK);
    CHECK(n_dfs == (int64_t)ids.size() && n_geom == 3 && n_wgs % 32 == 0);
    const int n_sl = geom[2];
    std::map<int, std::vector<std::pair<int32_t, int>>> seen;  // row group -> (block, filled slots)
    auto partitioned = [&](int ofs, int cnt, int n_full) {
        if (n_full < 0 || n_full > cnt || 2 * (int64_t)(ofs + cnt) > n_tiles) return false;
        for (int k = 0; k < cnt; ++k) {
            const int valid = (tiles[2 * (ofs + k) + 1] >> 20) & 31;
            if (k < n_full ? valid != 16 : (valid < 1 || valid > 15)) return false;
        }
        return true;
    };
    for (int64_t w = 0; w < n_wgs / 32; ++w) {
        const int32_t* wg = wgs.data() + 32 * w;
        CHECK(partitioned(wg[0], wg[1], wg[3] >> 8));
        for (int k = 0; k < 4; ++k) {
            const int32_t* it = wg + 4 + 6 * k;
            CHECK(partitioned(it[0], it[1], wg[28 + k]));
            CHECK(it[3] > 0 || it[1] == 0);
            for (int g = it[2]; g < it[2] + it[3]; ++g) {
                for (int j = wg[0]; j < wg[0] + wg[1]; ++j) {
                    const int meta = tiles[2 * j + 1];
                    if ((meta & 1023) <= g - wg[2] && g - wg[2] < ((meta >> 10) & 1023)) seen[g].push_back({tiles[2 * j], (meta >> 20) & 31});
                }
                for (int j = it[0]; j < it[0] + it[1]; ++j) {
                    const int meta = tiles[2 * j + 1];
                    if ((meta & 1023) <= g - it[2] && g - it[2] < ((meta >> 10) & 1023)) seen[g].push_back({tiles[2 * j], (meta >> 20) & 31});
                }
            }
        }
    }
    CHECK(seen.size() == ids.size() * (size_t)n_sl);
    std::set<int32_t> uniq;
    int64_t path_tokens = 0;
    std::vector<int32_t> tb(512);
    for (size_t rank = 0; rank < ids.size(); ++rank) {
        CHECK(dfs[rank] >= 0 && (size_t)dfs[rank] < ids.size());
        const apar_thread t = ids[dfs[rank]];
        int n = 0;
        int64_t L = 0;
        CHECK(apar_thread_block_table(p, t, tb.data(), (int)tb.size(), &n) == APAR_OK && apar_thread_len(p, t, &L) == APAR_OK);
        std::vector<int32_t> table(tb.begin(), tb.begin() + n);
        uniq.insert(table.begin(), table.end());
        path_tokens += L;
        const int32_t last = table.back();
        std::sort(table.begin(), table.end());
        for (int sl = 0; sl < n_sl; ++sl) {
            auto& got = seen[(int)rank * n_sl + sl];
            std::vector<int32_t> blocks;
            int64_t rows = 0;
            for (auto& bv : got) {
                blocks.push_back(bv.first), rows += bv.second;
                CHECK(bv.second == 16 || bv.first == last);
            }
            std::sort(blocks.begin(), blocks.end());
            CHECK(blocks == table && rows == L);
        }
    }
    apar_plan_info info{};
    CHECK(apar_last_plan_info(p, &info) == APAR_OK);
    CHECK(info.unique_blocks == (int64_t)uniq.size() && info.path_tokens == path_tokens && info.n_threads == (int64_t)ids.size());
    return 0;
}

// The device's copy of the plan tables, were only the ints rewritten that the library names as changed by a call
// that carried its plan over: kept the same way here and compared with the tables on the host after every call.
struct TablesOnDevice {
    std::vector<int32_t> wgs, tiles;
    int64_t carried = 0;
    int follow(apar_pool* p, int seed) {
        auto table = [&](int which, std::vector<int32_t>& out) {
            int64_t n = 0;
            apar_last_plan_export(p, which, nullptr, 0, &n);
            out.assign(n + 1, 0);
            const int rc = apar_last_plan_export(p, which, out.data(), n, &n);
            out.resize(n);
            return rc;
        };
        std::vector<int32_t> w, t, cw, ct;
        CHECK(table(APAR_PLAN_WORKGROUPS, w) == APAR_OK && table(APAR_PLAN_TILES, t) == APAR_OK);
        CHECK(table(APAR_PLAN_CHANGED_WORKGROUP_WORDS, cw) == APAR_OK && table(APAR_PLAN_CHANGED_TILE_WORDS, ct) == APAR_OK);
        int64_t built = 0, now = 0;
        apar_plan_counts(p, &built, &now);
        const bool was_carried = now > carried;
        carried = now;
        if (was_carried && !wgs.empty()) {
            CHECK(wgs.size() == w.size() && tiles.size() == t.size());
            for (int32_t i : cw) wgs[i] = w[i];
            for (int32_t i : ct) tiles[i] = t[i];
            CHECK(wgs == w && tiles == t);
        } else {
            CHECK(was_carried || (cw.empty() && ct.empty()));
            wgs = w, tiles = t;
        }
        return 0;
    }
};

static int64_t n_carried_total = 0;  // plans carried over by the decode loops of all sequences

static int pool_ops(int seed) {
    std::mt19937 rng(seed);
    auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
    const int groups[] = {1, 2, 4, 8};
    apar_pool_config cfg{};
    cfg.n_kv_heads = rnd(1, 2);
    cfg.n_q_heads = cfg.n_kv_heads * groups[rng() % 4];
    cfg.head_dim = 128;
    cfg.block_size = 16;
    cfg.dtype = rng() % 2 ? APAR_BF16 : APAR_F32;
    cfg.max_threads = rnd(8, 400);
    cfg.num_blocks = rnd(4, 300);
    apar_pool* p = nullptr;
    CHECK(apar_pool_create(&cfg, nullptr, 0, &p) == APAR_OK);
    CHECK(apar_set_write_checks(p, 1) == APAR_OK);
    std::vector<apar_thread> live;
    std::map<apar_thread, int64_t> len;
    auto stats_ok = [&](int seed) -> int {
        apar_stats st{};
        CHECK(apar_pool_stats(p, &st) == APAR_OK);
        CHECK(st.used_blocks + st.free_blocks == cfg.num_blocks && st.live_threads == (int64_t)live.size());
        std::map<int32_t, int> holders;
        std::vector<int32_t> tb(cfg.num_blocks + 1);
        for (apar_thread t : live) {
            int n = 0;
            int64_t L = 0;
            CHECK(apar_thread_block_table(p, t, tb.data(), (int)tb.size(), &n) == APAR_OK);
            CHECK(apar_thread_len(p, t, &L) == APAR_OK && L == len[t] && n == (L + 15) / 16);
            for (int i = 0; i < n; ++i) holders[tb[i]] += 1;
        }
        CHECK((int64_t)holders.size() == st.used_blocks);
        for (auto& kv : holders) {
            int32_t r = 0;
            CHECK(apar_block_refcount(p, kv.first, &r) == APAR_OK && r == kv.second);
        }
        return 0;
    };
    for (int step = 0; step < 300; ++step) {
        const int op = rnd(0, 10);
        apar_stats before{};
        apar_pool_stats(p, &before);
        int rc = APAR_OK;
        if (op == 0 || live.empty()) {
            apar_thread t = -1;
            rc = apar_thread_create(p, &t);
            CHECK(rc == APAR_OK || rc == APAR_ERR_THREAD_CAPACITY);
            if (rc == APAR_OK) live.push_back(t), len[t] = 0;
        } else if (op <= 2) {
            const apar_thread t = live[rng() % live.size()];
            const int n = rnd(0, 70);
            rc = apar_append_kv(p, t, nullptr, nullptr, n, nullptr);
            CHECK(rc == APAR_OK || rc == APAR_ERR_OUT_OF_BLOCKS);
            if (rc == APAR_OK) len[t] += n;
        } else if (op == 3) {
            const apar_thread t = live[rng() % live.size()];
            const int k = rnd(1, rng() % 5 == 0 ? 150 : 4);
            std::vector<apar_thread> kids(k);
            rc = apar_fork(p, t, k, kids.data());
            CHECK(rc == APAR_OK || rc == APAR_ERR_THREAD_CAPACITY);
            if (rc == APAR_OK)
                for (apar_thread c : kids) live.push_back(c), len[c] = len[t];
        } else if (op == 4) {
            const size_t i = rng() % live.size();
            CHECK(apar_free_thread(p, live[i]) == APAR_OK);
            CHECK(apar_free_thread(p, live[i]) == APAR_ERR_INVALID_THREAD);
            len.erase(live[i]);
            live.erase(live.begin() + i);
        } else if (op == 5) {  // one row per listed thread, repeats allowed
            std::vector<apar_thread> ids;
            for (int i = rnd(1, 60); i > 0; --i) ids.push_back(live[rng() % live.size()]);
            rc = apar_append_kv_batch(p, ids.data(), (int)ids.size(), nullptr, nullptr, nullptr);
            CHECK(rc == APAR_OK || rc == APAR_ERR_OUT_OF_BLOCKS);
            if (rc == APAR_OK)
                for (apar_thread t : ids) len[t] += 1;
        } else if (op == 6) {  // commit of a multi-candidate step over distinct threads
            std::vector<apar_thread> ids;
            for (apar_thread t : live)
                if (rng() % 2) ids.push_back(t);
            const int C = rnd(1, 8);
            std::vector<uint8_t> masks(ids.size());
            for (uint8_t& m : masks) m = (uint8_t)(rng() & ((1u << C) - 1));
            rc = apar_commit_candidates(p, ids.data(), (int)ids.size(), nullptr, nullptr, C, masks.data(), nullptr);
            CHECK(rc == APAR_OK || rc == APAR_ERR_OUT_OF_BLOCKS);
            if (rc == APAR_OK)
                for (size_t i = 0; i < ids.size(); ++i) len[ids[i]] += __builtin_popcount(masks[i]);
        } else if (op == 7) {  // plans over the threads that have rows
            std::vector<apar_thread> ids;
            for (apar_thread t : live)
                if (len[t] > 0 && rng() % 4) ids.push_back(t);
            apar_set_chunk_blocks(p, rnd(1, 40));
            apar_set_matrix_units(p, rnd(0, 2) * 32, rnd(1, 8));
            apar_set_inline_shared(p, (int)(rng() % 2));
            const int C = rnd(1, 8);
            rc = (C * (cfg.n_q_heads / cfg.n_kv_heads) <= 64 && rng() % 2)
                     ? apar_decode_attention_spec(p, nullptr, nullptr, nullptr, nullptr, C, ids.data(), (int)ids.size(), nullptr, nullptr)
                     : apar_decode_attention(p, nullptr, ids.data(), (int)ids.size(), nullptr, nullptr);
            CHECK(rc == APAR_OK);
            if (!ids.empty() && plan_covers_tables(p, ids, seed)) return 1;
            if (!ids.empty()) {
                int64_t n_out = 0;
                std::vector<int32_t> buf(1 << 20);
                for (int which = 0; which < 6; ++which) CHECK(apar_last_plan_export(p, which, buf.data(), (int64_t)buf.size(), &n_out) == APAR_OK);
                std::vector<int32_t> m(ids.size());
                for (size_t i = 0; i < ids.size(); ++i) m[i] = 1 + (int)(rng() % (unsigned)len[ids[i]]);
                rc = apar_prefill_attention(p, nullptr, ids.data(), m.data(), (int)ids.size(), nullptr, nullptr);
                CHECK(rc == APAR_OK);
            }
        } else if (op == 8) {
            // a decode loop: the same positions step after step, some threads replaced by a thread forked from them,
            // rows appended in between (one, a few, now and then enough for several blocks), forks that leave a
            // listed thread's last block shared; most of these plans are carried over, every one must cover the tables
            std::vector<apar_thread> ids;
            for (apar_thread t : live)
                if (len[t] > 0 && rng() % 4) ids.push_back(t);
            if (rng() % 8 == 0 && ids.size() > 1) ids.push_back(ids[0]);  // a thread listed twice
            apar_set_plan_reuse(p, rng() % 8 != 0);
            const int C = rnd(1, 3);
            const bool spec = C * (cfg.n_q_heads / cfg.n_kv_heads) <= 64 && rng() % 2;
            int64_t built0 = 0, carried0 = 0;
            apar_plan_counts(p, &built0, &carried0);
            TablesOnDevice on_device;
            on_device.carried = carried0;
            for (int round = 0; round < 12 && !ids.empty(); ++round) {
                for (size_t i = 0; i < ids.size(); ++i) {
                    const unsigned what = rng() % 64;
                    if (what == 0) {  // replaced by a child; the parent goes (unless it is listed elsewhere too)
                        apar_thread c = -1;
                        if (apar_fork(p, ids[i], 1, &c) != APAR_OK) continue;
                        live.push_back(c), len[c] = len[ids[i]];
                        if (std::count(ids.begin(), ids.end(), ids[i]) == 1 && rng() % 4) {
                            CHECK(apar_free_thread(p, ids[i]) == APAR_OK);
                            len.erase(ids[i]);
                            live.erase(std::find(live.begin(), live.end(), ids[i]));
                        }
                        ids[i] = c;
                    } else if (what == 1) {  // a fork that is not listed: the last block is shared from here on
                        apar_thread c = -1;
                        if (apar_fork(p, ids[i], 1, &c) == APAR_OK) live.push_back(c), len[c] = len[ids[i]];
                    } else if (what == 2) {
                        const int n = rnd(2, 40);
                        if (apar_append_kv(p, ids[i], nullptr, nullptr, n, nullptr) == APAR_OK) len[ids[i]] += n;
                    }
                }
                std::vector<apar_thread> distinct(ids);
                std::sort(distinct.begin(), distinct.end());
                distinct.erase(std::unique(distinct.begin(), distinct.end()), distinct.end());
                if (rng() % 3) {
                    if (apar_append_kv_batch(p, distinct.data(), (int)distinct.size(), nullptr, nullptr, nullptr) == APAR_OK)
                        for (apar_thread t : distinct) len[t] += 1;
                } else {
                    std::vector<uint8_t> masks(distinct.size());
                    for (uint8_t& m : masks) m = (uint8_t)(rng() & 7);
                    if (apar_commit_candidates(p, distinct.data(), (int)distinct.size(), nullptr, nullptr, 3, masks.data(), nullptr) == APAR_OK)
                        for (size_t i = 0; i < distinct.size(); ++i) len[distinct[i]] += __builtin_popcount(masks[i]);
                }
                rc = spec ? apar_decode_attention_spec(p, nullptr, nullptr, nullptr, nullptr, C, ids.data(), (int)ids.size(), nullptr, nullptr)
                          : apar_decode_attention(p, nullptr, ids.data(), (int)ids.size(), nullptr, nullptr);
                CHECK(rc == APAR_OK);
                if (plan_covers_tables(p, ids, seed) || on_device.follow(p, seed)) return 1;
            }
            int64_t built1 = 0, carried1 = 0;
            apar_plan_counts(p, &built1, &carried1);
            n_carried_total += carried1 - carried0;
            apar_set_plan_reuse(p, 1);
            rc = APAR_OK;
        } else {  // bad arguments must be refused and change nothing
            CHECK(apar_append_kv(p, 1 << 29, nullptr, nullptr, 3, nullptr) == APAR_ERR_INVALID_THREAD);
            CHECK(apar_fork(p, live[0], 0, nullptr) == APAR_ERR_INVALID_ARG);
            rc = APAR_ERR_INVALID_ARG;
        }
        if (rc != APAR_OK) {
            apar_stats after{};
            apar_pool_stats(p, &after);
            CHECK(after.used_blocks == before.used_blocks && after.live_threads == before.live_threads &&
                  after.threads_issued == before.threads_issued && after.cow_copies == before.cow_copies);
        }
        if (step % 25 == 0 && stats_ok(seed)) return 1;
    }
    if (stats_ok(seed)) return 1;
    CHECK(apar_pool_destroy(p) == APAR_OK);
    return 0;
}

static int serving(int seed) {
    std::mt19937 rng(seed);
    auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
    apar_pool_config cfg{};
    cfg.n_q_heads = cfg.n_kv_heads = 2;
    cfg.head_dim = 128;
    cfg.block_size = 16;
    cfg.dtype = APAR_BF16;
    cfg.max_threads = 1 << 20;
    cfg.num_blocks = rnd(24, 200);
    apar_pool* p = nullptr;
    CHECK(apar_pool_create(&cfg, nullptr, 0, &p) == APAR_OK);
    CHECK(apar_set_write_checks(p, 1) == APAR_OK);
    apar_server_config sc{rnd(1, 12), rnd(0, 4)};
    apar_server* sv = nullptr;
    CHECK(apar_server_create(p, &sc, &sv) == APAR_OK);
    const int n_req = rnd(1, 30);
    for (int r = 0; r < n_req; ++r) {
        std::vector<int32_t> prompt(rnd(1, 120));
        for (int32_t& x : prompt) x = rnd(0, 999);
        CHECK(apar_server_submit(sv, r, prompt.data(), (int)prompt.size()) == APAR_OK);
    }
    int finished = 0;
    std::vector<apar_server_seq> batch(4096);
    std::vector<int32_t> toks(1 << 16);
    for (int step = 0; step < 4000 && finished < n_req; ++step) {
        int32_t n_adm = 0;
        int64_t rows = 0;
        CHECK(apar_server_admit(sv, nullptr, nullptr, 1 << 20, nullptr, &n_adm, &rows) == APAR_OK);
        int nb = 0;
        CHECK(apar_server_batch(sv, batch.data(), (int)batch.size(), &nb) == APAR_OK);
        if (nb == 0) continue;
        std::vector<int32_t> sampled(nb);
        for (int i = 0; i < nb; ++i) {
            const unsigned u = rng() % 100;
            const bool can_fork = batch[i].group_size < 6 && batch[i].last_token != APAR_TOKEN_FORK;
            sampled[i] = (u < 6 && can_fork) ? APAR_TOKEN_FORK : (u < 10 || batch[i].length > 300) ? APAR_TOKEN_EOS : rnd(0, 999);
        }
        apar_server_step_info info{};
        const int rc = apar_server_step(sv, sampled.data(), nb, nullptr, nullptr, nullptr, &info);
        CHECK(rc == APAR_OK);
        for (;;) {
            int32_t rid = -1;
            int64_t nt = 0;
            apar_group_info gi{};
            CHECK(apar_server_pop_finished(sv, &rid, toks.data(), (int64_t)toks.size(), &nt, &gi) == APAR_OK);
            if (rid < 0) break;
            ++finished;
        }
        apar_stats st{};
        CHECK(apar_pool_stats(p, &st) == APAR_OK && st.used_blocks + st.free_blocks == cfg.num_blocks);
    }
    apar_server_stats ss{};
    CHECK(apar_server_get_stats(sv, &ss) == APAR_OK);
    CHECK(apar_server_destroy(sv) == APAR_OK);
    apar_stats st{};
    CHECK(apar_pool_stats(p, &st) == APAR_OK && st.used_blocks == 0 && st.live_threads == 0);
    CHECK(apar_pool_destroy(p) == APAR_OK);
    return 0;
}

int main(int argc, char** argv) {
    const int first = argc > 1 ? std::atoi(argv[1]) : 0, count = argc > 2 ? std::atoi(argv[2]) : 100;
    for (int seed = first; seed < first + count; ++seed)
        if (pool_ops(seed) || serving(seed)) return 1;
    if (count >= 20 && n_carried_total < count) {
        std::fprintf(stderr, "only %lld plans were carried over: the decode loops do not exercise it\n", (long long)n_carried_total);
        return 1;
    }
    std::printf("ok: %d sequences, %lld plans carried over\n", count, (long long)n_carried_total);
    return 0;
}
