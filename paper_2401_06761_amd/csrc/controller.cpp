// The decoding controller of APAR (Alg. 1) on top of the pool's C ABI: one
// sequence group per prompt, fork on a [Fork] token, forced [Child] token in the
// new thread, paragraph-node bookkeeping, release on [EOS], and Restore of the
// paragraph tree into one linear sequence.  It samples nothing: the caller runs
// the decode step over the unfinished sequences and hands in the tokens it drew.
// Everything here goes through the public calls of apar.h.
#include <algorithm>
#include <cstring>
#include <deque>
#include <new>
#include <vector>

#include "apar.h"

namespace {

struct Seq {
    apar_thread tid = -1;
    bool finished = false;
    int32_t last_token = 0;
    std::vector<int32_t> tokens;
    int32_t current_node = -1;
    int32_t parent = -1;     // sequence it was forked from
    int64_t fork_len = 0;    // tokens it shares with that parent (0 for the prompt sequence)
};

struct PNode {               // points at tokens[start:end] of its sequence (end < 0: to the end)
    int32_t seq;
    int64_t start, end;
    int32_t first_child, next_sibling;
};

}  // namespace

struct apar_group {
    apar_pool* pool = nullptr;
    std::vector<Seq> seqs;
    std::vector<PNode> nodes;
    int64_t prompt_len = 0;
    int64_t attended = 0, generated = 0, max_cached = 0, cached_now = 0, steps = 0;
};

namespace {

int32_t new_node(apar_group* g, int32_t seq, int64_t start) {
    g->nodes.push_back(PNode{seq, start, -1, -1, -1});
    return (int32_t)g->nodes.size() - 1;
}

// KV slots the group needs right now, counted in tokens: a sequence's own tokens
// (those past its fork point) are needed up to its length while it runs, and after
// it finished only as far as a still-needed child shares them.
int64_t cached_tokens(const apar_group* g) {
    const int n = (int)g->seqs.size();
    std::vector<int64_t> need(n, 0);
    std::vector<char> alive(n, 0);
    int64_t total = 0;
    for (int q = n - 1; q >= 0; --q) {  // children come after their parents
        const Seq& s = g->seqs[q];
        if (!s.finished) {
            alive[q] = 1;
            need[q] = (int64_t)s.tokens.size();
        }
        if (alive[q]) {
            total += std::max<int64_t>(0, need[q] - s.fork_len);
            if (s.parent >= 0) {
                alive[s.parent] = 1;
                if (g->seqs[s.parent].finished) need[s.parent] = std::max(need[s.parent], s.fork_len);
            }
        }
    }
    return total;
}

// One decoding step of Alg. 1 for a group, in three parts, so that several groups can share one batched append:
// prepare forks the sequences whose last token is [Fork] and lists the threads of the rows to append
// ([Child] row of a new thread, then the sampled token's row of its parent); commit does the bookkeeping
// of Alg. 1 once the rows are in; rollback releases the forked children when they are not.
struct StepPlan {
    std::vector<int32_t> active;     // indices of the unfinished sequences, creation order
    std::vector<apar_thread> kids;   // children forked by prepare, in order
    std::vector<apar_thread> rows;   // thread of every row to append, in order
};

int step_prepare(apar_group* g, const int32_t* sampled, int n, StepPlan& sp) {
    sp.active.clear(), sp.kids.clear(), sp.rows.clear();
    for (int q = 0; q < (int)g->seqs.size(); ++q)
        if (!g->seqs[q].finished) sp.active.push_back(q);
    if ((int)sp.active.size() != n) return APAR_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (sampled[i] == APAR_TOKEN_CHILD) return APAR_ERR_INVALID_ARG;  // injected, never sampled
    // fork first (Alg. 1: a sequence that ends in [Fork] spawns a copy of itself); undone if the rows do not fit
    for (int i = 0; i < n; ++i) {
        Seq& s = g->seqs[sp.active[i]];
        if (s.last_token == APAR_TOKEN_FORK) {
            apar_thread child;
            const int rc = apar_fork(g->pool, s.tid, 1, &child);
            if (rc != APAR_OK) {
                for (apar_thread c : sp.kids) (void)apar_free_thread(g->pool, c);
                sp.kids.clear();
                return rc;
            }
            sp.kids.push_back(child);
            sp.rows.push_back(child);  // the [Child] row
        }
        sp.rows.push_back(s.tid);      // the sampled token's row
    }
    return APAR_OK;
}

void step_rollback(apar_group* g, StepPlan& sp) {
    for (apar_thread c : sp.kids) (void)apar_free_thread(g->pool, c);
    sp.kids.clear();
}

// A sequence that ends in [Fork] gets a detail thread: the new sequence holds the parent's tokens and the
// forced [Child] token; the parent's open paragraph ends where the parent stands, the detail paragraph
// becomes its first child and what the parent writes next its next sibling (Alg. 1; Sec. 2.2 "Paragraph tree").
void attach_detail_thread(apar_group* g, int32_t parent, apar_thread child_tid) {
    const int32_t detail = (int32_t)g->seqs.size();
    {
        Seq d;
        d.tid = child_tid;
        d.parent = parent;
        d.fork_len = (int64_t)g->seqs[parent].tokens.size();
        d.tokens.reserve((size_t)d.fork_len + 64);
        d.tokens = g->seqs[parent].tokens;
        d.tokens.push_back(APAR_TOKEN_CHILD);
        d.last_token = APAR_TOKEN_CHILD;
        g->seqs.push_back(std::move(d));
    }
    const int64_t at = g->seqs[detail].fork_len;
    const int32_t below = new_node(g, detail, at + 1);  // after the [Child] token
    const int32_t after = new_node(g, parent, at);
    PNode& closed = g->nodes[g->seqs[parent].current_node];
    closed.end = at;
    closed.first_child = below;
    closed.next_sibling = after;
    g->seqs[detail].current_node = below;
    g->seqs[parent].current_node = after;
}

void step_commit(apar_group* g, const int32_t* sampled, const StepPlan& sp, apar_group_step_info* info) {
    const int n = (int)sp.active.size();
    size_t kid = 0;
    int n_finished = 0;
    for (int i = 0; i < n; ++i) {
        const int32_t q = sp.active[i];
        g->attended += (int64_t)g->seqs[q].tokens.size();  // the sampled token was predicted from the whole sequence
        g->generated += 1;
        if (g->seqs[q].last_token == APAR_TOKEN_FORK) attach_detail_thread(g, q, sp.kids[kid++]);
        Seq& s = g->seqs[q];
        s.tokens.push_back(sampled[i]);
        s.last_token = sampled[i];
        if (sampled[i] == APAR_TOKEN_EOS) {
            s.finished = true;
            (void)apar_free_thread(g->pool, s.tid);  // Alg. 1 ReleaseCache: only blocks no other thread holds go back
            ++n_finished;
        }
    }
    g->steps += 1;
    g->cached_now = cached_tokens(g);
    g->max_cached = std::max(g->max_cached, g->cached_now);
    if (info) {
        info->n_forked = (int32_t)sp.kids.size();
        info->n_finished = n_finished;
        info->n_rows_appended = (int32_t)sp.rows.size();
        info->n_unfinished = 0;
        for (const Seq& s : g->seqs) info->n_unfinished += s.finished ? 0 : 1;
    }
}

int64_t restore_tokens(const apar_group* g, int32_t* tokens_out, int64_t cap) {
    // Alg. 1 Restore: a node, then its first child's subtree, then its next sibling's
    int64_t n = 0;
    std::vector<int32_t> stack{0};
    while (!stack.empty()) {
        const int32_t id = stack.back();
        stack.pop_back();
        const PNode& nd = g->nodes[id];
        const std::vector<int32_t>& tok = g->seqs[nd.seq].tokens;
        const int64_t end = nd.end < 0 ? (int64_t)tok.size() : nd.end;
        for (int64_t i = nd.start; i < end; ++i) {
            if (n < cap) tokens_out[n] = tok[i];
            ++n;
        }
        if (nd.next_sibling >= 0) stack.push_back(nd.next_sibling);
        if (nd.first_child >= 0) stack.push_back(nd.first_child);
    }
    return n;
}

void fill_info(const apar_group* g, apar_group_info* out) {
    out->n_sequences = (int64_t)g->seqs.size();
    out->n_unfinished = 0;
    for (const Seq& s : g->seqs) out->n_unfinished += s.finished ? 0 : 1;
    out->n_nodes = (int64_t)g->nodes.size();
    out->steps = g->steps;
    out->prompt_tokens = g->prompt_len;
    out->generated_tokens = g->generated;
    out->attended_tokens = g->attended;
    out->cached_tokens = g->cached_now;
    out->max_cached_tokens = g->max_cached;
}

}  // namespace

extern "C" {

int apar_group_create(apar_pool* pool, const int32_t* prompt_tokens, int n_prompt, const void* k_dev,
                      const void* v_dev, void* hip_stream, apar_group** out) {
    if (!pool || !prompt_tokens || n_prompt < 1 || !out) return APAR_ERR_INVALID_ARG;
    *out = nullptr;
    apar_thread t;
    int rc = apar_thread_create(pool, &t);
    if (rc != APAR_OK) return rc;
    rc = apar_append_kv(pool, t, k_dev, v_dev, n_prompt, hip_stream);
    if (rc != APAR_OK) {
        (void)apar_free_thread(pool, t);
        return rc;
    }
    apar_group* g = new (std::nothrow) apar_group();
    if (!g) {
        (void)apar_free_thread(pool, t);
        return APAR_ERR_INVALID_ARG;
    }
    g->pool = pool;
    g->prompt_len = n_prompt;
    Seq s;
    s.tid = t;
    s.tokens.assign(prompt_tokens, prompt_tokens + n_prompt);
    s.last_token = prompt_tokens[n_prompt - 1];
    g->seqs.push_back(std::move(s));
    g->seqs[0].current_node = new_node(g, 0, n_prompt);  // the root paragraph starts where the prompt ends
    g->cached_now = g->max_cached = n_prompt;
    *out = g;
    return APAR_OK;
}

int apar_group_destroy(apar_group* g) {
    if (!g) return APAR_OK;
    int rc = APAR_OK;
    for (Seq& s : g->seqs)
        if (!s.finished) {
            const int r = apar_free_thread(g->pool, s.tid);
            if (r != APAR_OK) rc = r;
        }
    delete g;
    return rc;
}

int apar_group_unfinished(apar_group* g, apar_thread* threads_out, int cap, int* n_out) {
    if (!g || !n_out || cap < 0 || (cap > 0 && !threads_out)) return APAR_ERR_INVALID_ARG;
    int n = 0;
    for (const Seq& s : g->seqs)
        if (!s.finished) {
            if (n < cap) threads_out[n] = s.tid;
            ++n;
        }
    *n_out = n;
    return n <= cap ? APAR_OK : APAR_ERR_INVALID_ARG;
}

int apar_group_step(apar_group* g, const int32_t* sampled, int n, const void* k_dev, const void* v_dev,
                    void* hip_stream, apar_group_step_info* info) {
    if (!g || n < 0 || (n > 0 && !sampled)) return APAR_ERR_INVALID_ARG;
    StepPlan sp;
    int rc = step_prepare(g, sampled, n, sp);
    if (rc != APAR_OK) return rc;
    if (n == 0) {
        if (info) memset(info, 0, sizeof(*info));
        return APAR_OK;
    }
    rc = apar_append_kv_batch(g->pool, sp.rows.data(), (int)sp.rows.size(), k_dev, v_dev, hip_stream);
    if (rc != APAR_OK) {
        step_rollback(g, sp);
        return rc;
    }
    step_commit(g, sampled, sp, info);
    return APAR_OK;
}

int apar_group_restore(apar_group* g, int32_t* tokens_out, int64_t cap, int64_t* n_out) {
    if (!g || !n_out || cap < 0 || (cap > 0 && !tokens_out)) return APAR_ERR_INVALID_ARG;
    const int64_t n = restore_tokens(g, tokens_out, cap);
    *n_out = n;
    return n <= cap ? APAR_OK : APAR_ERR_INVALID_ARG;
}

int apar_group_get_info(apar_group* g, apar_group_info* out) {
    if (!g || !out) return APAR_ERR_INVALID_ARG;
    fill_info(g, out);
    return APAR_OK;
}

// ---------------------------------------------------------------------------
// Serving loop: a queue of requests over one pool, with admission control, early
// release (inside every group's step) and preemption when the pool runs dry.
// ---------------------------------------------------------------------------
struct apar_server {
    apar_pool* pool = nullptr;
    apar_server_config cfg{};
    struct Waiting {
        int32_t rid;
        std::vector<int32_t> prompt;
        int64_t order;  // submission order; a preempted request keeps its own
    };
    std::deque<Waiting> waiting;
    struct Running {
        int32_t rid;
        int64_t order;
        apar_group* g;
        std::vector<int32_t> prompt;  // kept for a restart after preemption
    };
    std::vector<Running> running;  // admission order
    struct Finished {
        int32_t rid;
        std::vector<int32_t> tokens;
        apar_group_info info;
    };
    std::deque<Finished> finished;
    apar_server_stats st{};
    int64_t next_order = 0;
    std::vector<StepPlan> plans;
    std::vector<apar_thread> batch_threads;
    std::vector<int32_t> batch_src;
};

static void server_note_usage(apar_server* s) {
    apar_stats ps;
    if (apar_pool_stats(s->pool, &ps) == APAR_OK) s->st.peak_used_blocks = std::max(s->st.peak_used_blocks, ps.used_blocks);
    s->st.peak_running = std::max<int64_t>(s->st.peak_running, (int64_t)s->running.size());
}

int apar_server_create(apar_pool* pool, const apar_server_config* cfg, apar_server** out) {
    if (!pool || !cfg || !out || cfg->max_running < 1 || cfg->watermark_blocks < 0) return APAR_ERR_INVALID_ARG;
    apar_server* s = new (std::nothrow) apar_server();
    if (!s) return APAR_ERR_INVALID_ARG;
    s->pool = pool;
    s->cfg = *cfg;
    *out = s;
    return APAR_OK;
}

int apar_server_destroy(apar_server* s) {
    if (!s) return APAR_OK;
    int rc = APAR_OK;
    for (auto& r : s->running) {
        const int e = apar_group_destroy(r.g);
        if (e != APAR_OK) rc = e;
    }
    delete s;
    return rc;
}

int apar_server_submit(apar_server* s, int32_t request_id, const int32_t* prompt_tokens, int n_prompt) {
    if (!s || !prompt_tokens || n_prompt < 1) return APAR_ERR_INVALID_ARG;
    apar_server::Waiting w;
    w.rid = request_id;
    w.prompt.assign(prompt_tokens, prompt_tokens + n_prompt);
    w.order = s->next_order++;
    s->waiting.push_back(std::move(w));
    s->st.n_submitted += 1;
    return APAR_OK;
}

int apar_server_admit(apar_server* s, const void* k_dev, const void* v_dev, int64_t rows_available, void* hip_stream,
                      int32_t* n_admitted_out, int64_t* rows_used_out) {
    if (!s || rows_available < 0) return APAR_ERR_INVALID_ARG;
    apar_stats ps;
    int rc = apar_pool_stats(s->pool, &ps);
    if (rc != APAR_OK) return rc;
    const bool dry = k_dev == nullptr && v_dev == nullptr;
    const int64_t row_bytes = ps.block_bytes / 16 / 2;  // one token's K (or V) row over all kv heads
    int32_t admitted = 0;
    int64_t used = 0;
    while (!s->waiting.empty() && (int)s->running.size() < s->cfg.max_running) {
        apar_server::Waiting& w = s->waiting.front();
        const int64_t n = (int64_t)w.prompt.size();
        const int64_t need = (n + 15) / 16;
        if ((rc = apar_pool_stats(s->pool, &ps)) != APAR_OK) return rc;
        // first come first served: the head of the queue waits until it fits, nobody overtakes it
        if (ps.free_blocks - need < s->cfg.watermark_blocks) break;
        if (used + n > rows_available) break;
        apar_group* g = nullptr;
        rc = apar_group_create(s->pool, w.prompt.data(), (int)n, dry ? nullptr : (const char*)k_dev + used * row_bytes,
                               dry ? nullptr : (const char*)v_dev + used * row_bytes, hip_stream, &g);
        if (rc == APAR_ERR_OUT_OF_BLOCKS || rc == APAR_ERR_THREAD_CAPACITY) break;
        if (rc != APAR_OK) return rc;
        apar_server::Running r;
        r.rid = w.rid;
        r.order = w.order;
        r.g = g;
        r.prompt = std::move(w.prompt);
        s->running.push_back(std::move(r));
        s->waiting.pop_front();
        used += n;
        ++admitted;
        s->st.n_admissions += 1;
    }
    server_note_usage(s);
    if (n_admitted_out) *n_admitted_out = admitted;
    if (rows_used_out) *rows_used_out = used;
    return APAR_OK;
}

int apar_server_batch(apar_server* s, apar_server_seq* out, int cap, int* n_out) {
    if (!s || !n_out || cap < 0 || (cap > 0 && !out)) return APAR_ERR_INVALID_ARG;
    int n = 0;
    for (const auto& r : s->running) {
        const apar_group* g = r.g;
        const int32_t size = (int32_t)g->seqs.size();
        for (int q = 0; q < size; ++q) {
            const Seq& sq = g->seqs[q];
            if (sq.finished) continue;
            if (n < cap) {
                apar_server_seq& e = out[n];
                e.request_id = r.rid;
                e.thread = sq.tid;
                e.seq_index = q;
                e.last_token = sq.last_token;
                e.length = (int64_t)sq.tokens.size();
                e.start_len = sq.parent < 0 ? g->prompt_len : sq.fork_len + 1;
                e.group_size = size;
                e.reserved = 0;
            }
            ++n;
        }
    }
    *n_out = n;
    return n <= cap ? APAR_OK : APAR_ERR_INVALID_ARG;
}

int apar_server_step(apar_server* s, const int32_t* sampled, int n, const void* k_dev, const void* v_dev,
                     void* hip_stream, apar_server_step_info* info) {
    if (!s || n < 0 || (n > 0 && !sampled)) return APAR_ERR_INVALID_ARG;
    if (info) memset(info, 0, sizeof(*info));
    // each running request's slice of `sampled` and of the rows in k_dev, v_dev
    const size_t n_run = s->running.size();
    std::vector<int32_t> tok_ofs(n_run + 1, 0), row_ofs(n_run + 1, 0);
    for (size_t r = 0; r < n_run; ++r) {
        const apar_group* g = s->running[r].g;
        int32_t unfinished = 0, forking = 0;
        for (const Seq& sq : g->seqs)
            if (!sq.finished) {
                ++unfinished;
                forking += sq.last_token == APAR_TOKEN_FORK ? 1 : 0;
            }
        tok_ofs[r + 1] = tok_ofs[r] + unfinished;
        row_ofs[r + 1] = row_ofs[r] + unfinished + forking;
    }
    if (tok_ofs[n_run] != n) return APAR_ERR_INVALID_ARG;
    s->plans.resize(n_run);
    size_t n_live = n_run;  // requests [0, n_live) take part; the ones after them were preempted in this call
    // put the preempted requests back, oldest first at the head
    auto requeue = [&]() {
        for (size_t r = n_run; r-- > n_live;) {
            apar_server::Waiting w;
            w.rid = s->running[r].rid;
            w.order = s->running[r].order;
            w.prompt = std::move(s->running[r].prompt);
            s->waiting.push_front(std::move(w));
        }
        s->running.resize(n_live);
        std::stable_sort(s->waiting.begin(), s->waiting.end(),
                         [](const apar_server::Waiting& a, const apar_server::Waiting& b) { return a.order < b.order; });
    };
    for (;;) {
        s->batch_threads.clear();
        s->batch_src.clear();
        int rc = APAR_OK;
        size_t prepared = 0;
        for (; prepared < n_live; ++prepared) {
            rc = step_prepare(s->running[prepared].g, sampled + tok_ofs[prepared],
                              tok_ofs[prepared + 1] - tok_ofs[prepared], s->plans[prepared]);
            if (rc != APAR_OK) break;
            const StepPlan& sp = s->plans[prepared];
            for (size_t i = 0; i < sp.rows.size(); ++i) {
                s->batch_threads.push_back(sp.rows[i]);
                s->batch_src.push_back(row_ofs[prepared] + (int32_t)i);
            }
        }
        if (rc == APAR_OK && !s->batch_threads.empty())
            rc = apar_append_kv_gather(s->pool, s->batch_threads.data(), s->batch_src.data(),
                                       (int)s->batch_threads.size(), k_dev, v_dev, hip_stream);
        if (rc == APAR_OK) break;
        for (size_t r = 0; r < prepared; ++r) step_rollback(s->running[r].g, s->plans[r]);
        // A request that does not fit the pool even when it runs alone can never finish: requeueing it would
        // admit it again (its prompt fits) and replay the same overflow for ever.  It stays where it is and the
        // caller gets the error.
        if (rc != APAR_ERR_OUT_OF_BLOCKS || n_live <= 1) {
            requeue();
            return rc;
        }
        // the pool cannot hold this step: the most recently admitted request gives way (it is released
        // and goes back to the head of the queue, to start again from its prompt)
        apar_server::Running& victim = s->running[n_live - 1];
        (void)apar_group_destroy(victim.g);
        victim.g = nullptr;
        --n_live;
        s->st.n_preemptions += 1;
        if (info) info->n_preempted += 1;
    }
    requeue();
    // bookkeeping of Alg. 1 for everyone who stayed; early release happens in there
    int64_t batch = 0;
    for (size_t r = 0; r < n_live; ++r) {
        apar_group_step_info gi;
        step_commit(s->running[r].g, sampled + tok_ofs[r], s->plans[r], &gi);
        batch += tok_ofs[r + 1] - tok_ofs[r];
        if (info) {
            info->n_forked += gi.n_forked;
            info->n_finished_sequences += gi.n_finished;
            info->n_rows_appended += gi.n_rows_appended;
        }
    }
    s->st.steps += 1;
    s->st.generated_tokens += batch;
    s->st.batch_sequences_total += batch;
    s->st.peak_threads = std::max(s->st.peak_threads, batch);
    server_note_usage(s);  // the peak is reached before the finished requests are collected
    // completed requests leave, in admission order
    size_t keep = 0;
    for (size_t r = 0; r < n_live; ++r) {
        apar_group* g = s->running[r].g;
        bool done = true;
        for (const Seq& sq : g->seqs) done = done && sq.finished;
        if (!done) {
            if (keep != r) s->running[keep] = std::move(s->running[r]);
            ++keep;
            continue;
        }
        apar_server::Finished f;
        f.rid = s->running[r].rid;
        f.tokens.resize((size_t)restore_tokens(g, nullptr, 0));
        (void)restore_tokens(g, f.tokens.data(), (int64_t)f.tokens.size());
        fill_info(g, &f.info);
        s->finished.push_back(std::move(f));
        (void)apar_group_destroy(g);
        s->st.n_finished += 1;
        if (info) info->n_finished_requests += 1;
    }
    s->running.resize(keep);
    if (info) info->n_running = (int32_t)keep;
    return APAR_OK;
}

int apar_server_pop_finished(apar_server* s, int32_t* request_id_out, int32_t* tokens_out, int64_t cap,
                             int64_t* n_tokens_out, apar_group_info* info_out) {
    if (!s || !request_id_out || !n_tokens_out || cap < 0 || (cap > 0 && !tokens_out)) return APAR_ERR_INVALID_ARG;
    if (s->finished.empty()) {
        *request_id_out = -1;
        *n_tokens_out = 0;
        return APAR_OK;
    }
    apar_server::Finished& f = s->finished.front();
    *request_id_out = f.rid;
    *n_tokens_out = (int64_t)f.tokens.size();
    if (cap < (int64_t)f.tokens.size()) return APAR_ERR_INVALID_ARG;  // the request stays at the head
    if (!f.tokens.empty()) memcpy(tokens_out, f.tokens.data(), f.tokens.size() * sizeof(int32_t));
    if (info_out) *info_out = f.info;
    s->finished.pop_front();
    return APAR_OK;
}

int apar_server_get_stats(apar_server* s, apar_server_stats* out) {
    if (!s || !out) return APAR_ERR_INVALID_ARG;
    *out = s->st;
    out->n_waiting = (int64_t)s->waiting.size();
    out->n_running = (int64_t)s->running.size();
    return APAR_OK;
}

}  // extern "C"
