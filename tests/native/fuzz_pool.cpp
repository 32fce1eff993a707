// Memory-safety fuzz of the library's host side on bookkeeping-only pools (no GPU): allocator, copy-on-write,
// batched appends, candidate commits, plans, the Algorithm 1 controller and the serving loop, driven by random
// operation sequences on pools small enough to run out of blocks.  Built by tests/test_library_host.py as
// plain host C++ with the address and undefined-behaviour sanitizers; the kernels' launchers are stubs (a
// bookkeeping-only pool never calls them).  Checks: statuses are the documented ones, a failed call leaves the
// counters as they were, used + free blocks = pool size, refcounts equal the number of live holders.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <vector>

#include "apar_internal.hpp"

namespace apar {
hipError_t fixed_workspace_of_device(int, char** out) { static char nothing[256]; *out = nothing; return hipSuccess; }
hipError_t launch_append_rows(const Shape&, void*, const void*, const void*, const int32_t*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_block_copies(const Shape&, void*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_seal_blocks(const Shape&, void*, const int32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_read_rows(const Shape&, const void*, const int32_t*, int, void*, void*, hipStream_t) { std::abort(); }
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
        const int op = rnd(0, 9);
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
            if (!ids.empty()) {
                int64_t n_out = 0;
                std::vector<int32_t> buf(1 << 20);
                for (int which = 0; which < 6; ++which) CHECK(apar_last_plan_export(p, which, buf.data(), (int64_t)buf.size(), &n_out) == APAR_OK);
                std::vector<int32_t> m(ids.size());
                for (size_t i = 0; i < ids.size(); ++i) m[i] = 1 + (int)(rng() % (unsigned)len[ids[i]]);
                rc = apar_prefill_attention(p, nullptr, ids.data(), m.data(), (int)ids.size(), nullptr, nullptr);
                CHECK(rc == APAR_OK);
            }
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
    std::printf("ok: %d sequences\n", count);
    return 0;
}
