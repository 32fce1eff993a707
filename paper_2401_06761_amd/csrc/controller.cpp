// The decoding controller of APAR (Alg. 1) on top of the pool's C ABI: one
// sequence group per prompt, fork on a [Fork] token, forced [Child] token in the
// new thread, paragraph-node bookkeeping, release on [EOS], and Restore of the
// paragraph tree into one linear sequence.  It samples nothing: the caller runs
// the decode step over the unfinished sequences and hands in the tokens it drew.
// Everything here goes through the public calls of apar.h.
#include <algorithm>
#include <cstring>
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
    std::vector<apar_thread> batch;
    std::vector<int32_t> forking;
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
    g->seqs[0].current_node = new_node(g, 0, n_prompt);  // r <- PNode(p, p.len)
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
    std::vector<int32_t> active;
    for (int q = 0; q < (int)g->seqs.size(); ++q)
        if (!g->seqs[q].finished) active.push_back(q);
    if ((int)active.size() != n) return APAR_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (sampled[i] == APAR_TOKEN_CHILD) return APAR_ERR_INVALID_ARG;  // injected, never sampled
    if (n == 0) {
        if (info) memset(info, 0, sizeof(*info));
        return APAR_OK;
    }
    // fork first (Alg. 1: s' <- s when s.last_token is [Fork]); undo them if the rows do not fit
    g->forking.clear();
    g->batch.clear();
    std::vector<apar_thread> kids;
    int rc = APAR_OK;
    for (int i = 0; i < n && rc == APAR_OK; ++i) {
        Seq& s = g->seqs[active[i]];
        if (s.last_token == APAR_TOKEN_FORK) {
            apar_thread child;
            rc = apar_fork(g->pool, s.tid, 1, &child);
            if (rc != APAR_OK) break;
            kids.push_back(child);
            g->forking.push_back(i);
            g->batch.push_back(child);  // the [Child] row
        }
        g->batch.push_back(s.tid);      // the sampled token's row
    }
    if (rc == APAR_OK)
        rc = apar_append_kv_batch(g->pool, g->batch.data(), (int)g->batch.size(), k_dev, v_dev, hip_stream);
    if (rc != APAR_OK) {
        for (apar_thread c : kids) (void)apar_free_thread(g->pool, c);
        return rc;
    }
    // commit: the bookkeeping of Alg. 1
    size_t kid = 0;
    int n_finished = 0;
    for (int i = 0; i < n; ++i) {
        const int32_t q = active[i];
        g->attended += (int64_t)g->seqs[q].tokens.size();  // predicting x attended to all of s
        g->generated += 1;
        if (g->seqs[q].last_token == APAR_TOKEN_FORK) {
            Seq c;
            c.tid = kids[kid++];
            c.tokens = g->seqs[q].tokens;
            c.tokens.push_back(APAR_TOKEN_CHILD);
            c.last_token = APAR_TOKEN_CHILD;
            c.parent = q;
            c.fork_len = (int64_t)g->seqs[q].tokens.size();
            const int32_t cq = (int32_t)g->seqs.size();
            g->seqs.push_back(std::move(c));
            Seq& s = g->seqs[q];
            const int32_t n_sib = new_node(g, q, (int64_t)s.tokens.size());
            const int32_t n_kid = new_node(g, cq, (int64_t)g->seqs[cq].tokens.size());
            PNode& cur = g->nodes[s.current_node];
            cur.end = (int64_t)s.tokens.size();
            cur.next_sibling = n_sib;
            cur.first_child = n_kid;
            s.current_node = n_sib;
            g->seqs[cq].current_node = n_kid;
        }
        Seq& s = g->seqs[q];
        s.tokens.push_back(sampled[i]);
        s.last_token = sampled[i];
        if (sampled[i] == APAR_TOKEN_EOS) {
            s.finished = true;
            (void)apar_free_thread(g->pool, s.tid);  // ReleaseCache(s)
            ++n_finished;
        }
    }
    g->steps += 1;
    g->cached_now = cached_tokens(g);
    g->max_cached = std::max(g->max_cached, g->cached_now);
    if (info) {
        info->n_forked = (int32_t)kids.size();
        info->n_finished = n_finished;
        info->n_rows_appended = (int32_t)g->batch.size();
        info->n_unfinished = 0;
        for (const Seq& s : g->seqs) info->n_unfinished += s.finished ? 0 : 1;
    }
    return APAR_OK;
}

int apar_group_restore(apar_group* g, int32_t* tokens_out, int64_t cap, int64_t* n_out) {
    if (!g || !n_out || cap < 0 || (cap > 0 && !tokens_out)) return APAR_ERR_INVALID_ARG;
    // Restore(r): node, then its first child's subtree, then its next sibling's
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
    *n_out = n;
    return n <= cap ? APAR_OK : APAR_ERR_INVALID_ARG;
}

int apar_group_get_info(apar_group* g, apar_group_info* out) {
    if (!g || !out) return APAR_ERR_INVALID_ARG;
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
    return APAR_OK;
}

}  // extern "C"
