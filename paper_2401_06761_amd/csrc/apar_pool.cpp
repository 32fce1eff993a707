// Host side of libapar: the C ABI, the block/refcount/fork bookkeeping, the
// plan builder that groups threads by the blocks they share, and the staging of
// small tables to the device.  Every device step runs in the HIP kernels; this
// file only decides which blocks they touch.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "apar_internal.hpp"
#include "plan.hpp"

using namespace apar;

namespace {

thread_local std::string g_last_hip_error;

bool hip_ok(hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return false;
}
#define HIP_TRY(expr)                                  \
    do {                                               \
        if (!hip_ok((expr), #expr)) return APAR_ERR_HIP; \
    } while (0)

struct Thread {
    bool live = false;
    int32_t forked_from = -1;  // the thread it was forked from (kept after either is released)
    int64_t len = 0;
    std::vector<int32_t> table;
};

// A pinned host buffer and its device twin, reused round-robin.  The event marks
// the last device work that read the pair, so a slot is only rewritten after it.
struct StageSlot {
    char* host = nullptr;
    char* dev = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;   // recorded after the kernels that read the slot
    hipEvent_t up = nullptr;   // recorded after the slot's upload
    bool pending = false;
};
constexpr int kStageSlots = 4;
constexpr size_t kCopyStreamMinBytes = 256 << 10;  // uploads from this size on run on the pool's copy stream

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr, c = nullptr;  // a..b first kernel(s), b..c second (c may be null)
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr size_t kFixedPlanBytes = (size_t)APAR_FIXED_PLAN_BYTES;
constexpr size_t kFixedPartBytes = (size_t)APAR_FIXED_PARTIAL_BYTES;

}  // namespace

struct apar_pool {
    apar_pool_config cfg{};
    Shape shape{};
    char* kv = nullptr;
    int device = 0;
    bool dry_run = false;  // bookkeeping and planning only: no device memory, nothing is launched

    std::vector<int32_t> ref;
    std::vector<int32_t> free_stack;
    std::vector<Thread> threads;  // index = thread id
    int64_t live_threads = 0;
    int64_t cow_copies = 0;

    // plan builder scratch (pool sized, kept clean between calls)
    std::vector<int32_t> seg_of;  // segment that starts at each block, -1 if none
    int max_unit_tiles = 512;  // longest tile list given to one wavefront
    int prefill_kernel = APAR_PREFILL_AUTO;
    // stand-alone segments with at least this many query rows and blocks run as matrix units (bf16 pools)
    int matrix_min_rows = 256, matrix_min_blocks = 128;
    bool inline_shared = true;  // subtrees with too many rows are cut by rank into direct units instead of leaving partial results
    bool check_writes = false;  // verify before every launch that no destination block is shared
    int last_prefill_kernel = 0;  // which kernel the most recent prefill call ran (APAR_PREFILL_ROW_TILES / _MATRIX)
    std::vector<PlanThreadView> views;
    std::vector<PrefillThreadView> prefill_views;
    std::vector<PrefillWg> prefill_wgs;
    std::vector<int32_t> prefill_tables;
    std::vector<int32_t> scratch_codes, scratch_copies, scratch_seals, scratch_commit_src;
    std::vector<apar_thread> scratch_commit_ids;
    apar_plan_info last_plan{};
    PlanHost plan;  // the last plan, kept for the next call to carry over, for reuse of its storage and for inspection
    // the call that plan was made or last carried over for: its listed threads, its parameters, and how many
    // threads the pool had ever created by then (a thread with an id from there on was forked since)
    std::vector<apar_thread> plan_ids;
    PlanParams plan_prm{};
    size_t plan_threads_then = 0;
    int64_t plan_copies_then = 0;  // copy-on-write copies the pool had made by then
    bool plan_reuse = true;
    int64_t n_plans_built = 0, n_plans_carried = 0;
    int32_t plan_geom[3] = {1, 1, 1};  // rows per thread, rows per slice, slices of the last plan

    StageSlot stage[kStageSlots];
    int next_slot = 0;
    size_t stage_want = 0;  // the largest staging request so far
    // The staging slot whose device half holds the tables of `plan`, as long as that is so: a call that carries
    // the plan over rewrites the changed words there instead of staging every table again.  Kept out of the
    // rotation meanwhile.  resident_behind: the host tables have moved on and the slot has not caught up yet
    // (set while a call is between the two; a call that fails there leaves it set and the slot is dropped).
    StageSlot* resident = nullptr;
    size_t resident_bytes = 0;
    bool resident_behind = false;
    PartialBuf part{};
    size_t part_slots_cap = 0;
    ClassStreams class_streams;
    hipStream_t copy_stream = nullptr;  // uploads of plans and row codes run here, beside the caller's stream

    // apar_decode_attention_fixed: this device's copy of the static workspace, a pinned host buffer the plan
    // is staged in, and the event after its upload; all three obtained at pool creation
    char* fixed_dev = nullptr;
    char* fixed_host = nullptr;
    hipEvent_t fixed_up = nullptr;
    bool fixed_pending = false;

    bool profiling = false;
    std::vector<EventPair> decode_events, append_events;
    std::vector<hipEvent_t> spare_events;
    std::vector<float> last_attention_ms;  // per call, from the last profile read
    double plan_host_ms = 0.0, host_wait_ms = 0.0, wait_in_call_ms = 0.0;
    int64_t n_decode_calls = 0, n_append_calls = 0;
};

namespace {

struct DeviceGuard {
    int prev = 0;
    bool switched = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) switched = (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard() {
        if (switched) (void)hipSetDevice(prev);
    }
};

Thread* live_thread(apar_pool* p, apar_thread t) {
    if (t < 0 || (size_t)t >= p->threads.size() || !p->threads[t].live) return nullptr;
    return &p->threads[t];
}

int32_t pop_block(apar_pool* p) {
    int32_t b = p->free_stack.back();
    p->free_stack.pop_back();
    p->ref[b] = 1;
    return b;
}

int acquire_stage(apar_pool* p, size_t bytes, StageSlot** out) {
    if (&p->stage[p->next_slot] == p->resident) p->next_slot = (p->next_slot + 1) % kStageSlots;
    StageSlot& s = p->stage[p->next_slot];
    p->next_slot = (p->next_slot + 1) % kStageSlots;
    if (s.pending) {
        const auto w0 = std::chrono::steady_clock::now();
        HIP_TRY(hipEventSynchronize(s.ev));
        s.pending = false;
        p->wait_in_call_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - w0).count();
        if (p->profiling) p->host_wait_ms += p->wait_in_call_ms;
    }
    if (!s.ev) HIP_TRY(hipEventCreateWithFlags(&s.ev, hipEventDisableTiming));
    // Growing a slot frees device memory, which waits for the GPU to drain: a slot grows to what the largest
    // request so far would need, not just to this one, so that the slots of a loop whose calls alternate
    // between small and large tables (row codes, plan updates) stop growing after one round.
    p->stage_want = std::max(p->stage_want, bytes);
    if (s.cap < bytes) {
        bytes = p->stage_want;
        if (s.host) HIP_TRY(hipHostFree(s.host));
        if (s.dev) HIP_TRY(hipFree(s.dev));
        s.host = s.dev = nullptr;
        s.cap = 0;
        size_t cap = align_up(std::max(bytes + bytes / 2, (size_t)1 << 20), 4096);
        HIP_TRY(hipHostMalloc((void**)&s.host, cap, hipHostMallocDefault));
        HIP_TRY(hipMalloc((void**)&s.dev, cap));
        s.cap = cap;
    }
    *out = &s;
    return APAR_OK;
}

// Uploads the first `bytes` of a staging slot on the pool's own copy stream and makes the caller's stream wait
// for it: the copy then runs beside whatever the caller's stream is still busy with (the previous step's
// attention, typically) instead of queueing behind it.  The slot is free by construction: acquire_stage waited
// for the kernels that last read it.
int upload(apar_pool* p, StageSlot* s, size_t bytes, hipStream_t st) {
    // Small tables go on the caller's stream: the hop to the copy stream and back costs more than it hides when a
    // step is a few launches long (a serving loop at a few hundred threads: 0.18 ms per step with the hop, 0.12 without).
    if (bytes < kCopyStreamMinBytes) {
        HIP_TRY(hipMemcpyAsync(s->dev, s->host, bytes, hipMemcpyHostToDevice, st));
        return APAR_OK;
    }
    if (!p->copy_stream) HIP_TRY(hipStreamCreateWithFlags(&p->copy_stream, hipStreamNonBlocking));
    if (!s->up) HIP_TRY(hipEventCreateWithFlags(&s->up, hipEventDisableTiming));
    HIP_TRY(hipMemcpyAsync(s->dev, s->host, bytes, hipMemcpyHostToDevice, p->copy_stream));
    HIP_TRY(hipEventRecord(s->up, p->copy_stream));
    HIP_TRY(hipStreamWaitEvent(st, s->up, 0));
    return APAR_OK;
}

int new_event(apar_pool* p, hipEvent_t* ev) {
    if (!p->spare_events.empty()) {
        *ev = p->spare_events.back();
        p->spare_events.pop_back();
        return APAR_OK;
    }
    HIP_TRY(hipEventCreate(ev));
    return APAR_OK;
}

// Where token slot `pos` of a thread lives: block * 16 + slot.
inline int32_t slot_code(const Thread& t, int64_t pos) {
    return t.table[pos / kBlockTokens] * kBlockTokens + (int32_t)(pos % kBlockTokens);
}

// Advances one thread by one token following the allocator policy; the caller
// has already made sure enough free blocks exist.
inline int32_t append_one(apar_pool* p, Thread& t, std::vector<int32_t>& copies, std::vector<int32_t>& seals) {
    const int slot = (int)(t.len % kBlockTokens);
    if (slot == 0) {
        t.table.push_back(pop_block(p));
    } else {
        const int32_t tail = t.table.back();
        if (p->ref[tail] > 1) {  // shared, partly filled tail: copy on write
            const int32_t fresh = pop_block(p);
            copies.push_back(tail);
            copies.push_back(fresh);
            p->ref[tail] -= 1;
            t.table.back() = fresh;
            p->cow_copies += 1;
        }
    }
    const int32_t code = t.table.back() * kBlockTokens + slot;
    if (slot == kBlockTokens - 1) seals.push_back(t.table.back());  // the block is full after this row
    t.len += 1;
    return code;
}

// Write check (apar_set_write_checks): every block about to be written - appended rows, destinations of
// copy-on-write copies, blocks about to be re-laid-out - must be held by exactly one thread.
int writes_are_private(const apar_pool* p, const std::vector<int32_t>& codes, const std::vector<int32_t>& copies,
                       const std::vector<int32_t>& seals) {
    for (int32_t c : codes)
        if (p->ref[c / kBlockTokens] != 1) return APAR_ERR_INTERNAL;
    for (size_t i = 0; i + 1 < copies.size(); i += 2)
        if (p->ref[copies[i + 1]] != 1 || copies[i] == copies[i + 1]) return APAR_ERR_INTERNAL;
    for (int32_t b : seals)
        if (p->ref[b] != 1) return APAR_ERR_INTERNAL;
    return APAR_OK;
}

// src_rows (may be null): which row of k, v each appended row is taken from.
int run_append(apar_pool* p, const std::vector<int32_t>& codes, const std::vector<int32_t>& copies,
               const std::vector<int32_t>& seals, const std::vector<int32_t>* src_rows, const void* k, const void* v,
               hipStream_t st) {
    const size_t copy_bytes = align_up(copies.size() * sizeof(int32_t), 256);
    const size_t code_bytes = align_up(codes.size() * sizeof(int32_t), 256);
    const size_t seal_bytes = align_up(seals.size() * sizeof(int32_t), 256);
    const size_t src_bytes = src_rows ? src_rows->size() * sizeof(int32_t) : 0;
    const size_t total = copy_bytes + code_bytes + seal_bytes + src_bytes;
    StageSlot* s = nullptr;
    int rc = acquire_stage(p, total, &s);
    if (rc != APAR_OK) return rc;
    if (!copies.empty()) memcpy(s->host, copies.data(), copies.size() * sizeof(int32_t));
    memcpy(s->host + copy_bytes, codes.data(), codes.size() * sizeof(int32_t));
    if (!seals.empty()) memcpy(s->host + copy_bytes + code_bytes, seals.data(), seals.size() * sizeof(int32_t));
    if (src_bytes) memcpy(s->host + copy_bytes + code_bytes + seal_bytes, src_rows->data(), src_bytes);
    if ((rc = upload(p, s, total, st)) != APAR_OK) return rc;
    EventPair ev;
    if (p->profiling) {
        if ((rc = new_event(p, &ev.a)) != APAR_OK || (rc = new_event(p, &ev.b)) != APAR_OK) return rc;
        HIP_TRY(hipEventRecord(ev.a, st));
    }
    if (!copies.empty())
        HIP_TRY(launch_block_copies(p->shape, p->kv, (const int32_t*)s->dev, (int)(copies.size() / 2), st));
    HIP_TRY(launch_append_rows(p->shape, p->kv, k, v, (const int32_t*)(s->dev + copy_bytes),
                               src_bytes ? (const int32_t*)(s->dev + copy_bytes + code_bytes + seal_bytes) : nullptr,
                               (int)codes.size(), st));
    if (!seals.empty())
        HIP_TRY(launch_seal_blocks(p->shape, p->kv, (const int32_t*)(s->dev + copy_bytes + code_bytes), (int)seals.size(), st));
    if (p->profiling) {
        HIP_TRY(hipEventRecord(ev.b, st));
        p->append_events.push_back(ev);
        p->n_append_calls += 1;
    }
    HIP_TRY(hipEventRecord(s->ev, st));
    s->pending = true;
    return APAR_OK;
}

bool same_params(const PlanParams& a, const PlanParams& b) {
    return a.rows_per_thread == b.rows_per_thread && a.max_unit_tiles == b.max_unit_tiles && a.allow_direct == b.allow_direct &&
           a.fuse == b.fuse && a.inline_shared == b.inline_shared && a.matrix_min_rows == b.matrix_min_rows &&
           a.matrix_min_blocks == b.matrix_min_blocks;
}

// fixed: the plan and the partial results go to the device's static workspace, nothing is allocated, no
// stream or event is created and profiling is off for the call.
int decode_common(apar_pool* p, const void* q, const void* cand_k, const void* cand_v, const uint8_t* mask,
                  int n_cand, const apar_thread* ids, int n, void* out, void* stream, bool spec, bool fixed = false) {
    if (!p || n < 0) return APAR_ERR_INVALID_ARG;
    if (fixed && (p->dry_run || !p->fixed_dev || !p->fixed_host)) return APAR_ERR_INVALID_ARG;
    if (n == 0) return APAR_OK;
    if (!ids) return APAR_ERR_INVALID_ARG;
    if (spec && (n_cand < 1 || n_cand > 8)) return APAR_ERR_INVALID_ARG;
    if (p->dry_run) {
        if (q || out || cand_k || cand_v || mask) return APAR_ERR_INVALID_ARG;
    } else {
        if (!q || !out) return APAR_ERR_INVALID_ARG;
        if (spec && (!cand_k || !cand_v || !mask)) return APAR_ERR_INVALID_ARG;
    }
    const auto t0 = std::chrono::steady_clock::now();
    p->wait_in_call_ms = 0.0;

    p->views.resize(n);
    for (int i = 0; i < n; ++i) {
        if (i + 16 < n && ids[i + 16] >= 0 && (size_t)ids[i + 16] < p->threads.size()) __builtin_prefetch(&p->threads[ids[i + 16]]);
        Thread* t = live_thread(p, ids[i]);
        if (!t) return APAR_ERR_INVALID_THREAD;
        if (t->len == 0) return APAR_ERR_INVALID_ARG;
        p->views[i] = PlanThreadView{t->table.data(), (int32_t)t->table.size(), t->len};
    }
    PlanHost& ph = p->plan;
    PlanParams prm;
    prm.rows_per_thread = n_cand * p->shape.group;
    prm.max_unit_tiles = p->max_unit_tiles;
    prm.allow_direct = true;
    prm.fuse = true;
    // (the 32x32 kernels read bf16 tiles only)
    prm.matrix_min_rows = (p->shape.dtype == APAR_BF16 && !p->shape.fp8_sealed) ? p->matrix_min_rows : 0;
    prm.matrix_min_blocks = p->matrix_min_blocks;
    prm.inline_shared = p->inline_shared;
    // Decode calls of a loop list the same threads step after step - each a few rows longer, a few replaced
    // by a thread forked from them - and the plan of the previous call then only needs its tails brought up
    // to date.  A table never changes before its last block, and a thread forked since the previous call
    // started from a copy of its parent's table as it was then or later, so "position by position the same
    // thread or one forked from it since" is all that has to hold for patch_plan to apply.
    bool carried = false;
    if (p->plan_reuse && ph.reusable && (size_t)n == p->plan_ids.size() && same_params(prm, p->plan_prm)) {
        bool same = true;
        for (int i = 0; i < n && same; ++i) {
            int32_t t = ids[i];
            while (t != p->plan_ids[i] && t >= 0 && (size_t)t >= p->plan_threads_then) t = p->threads[t].forked_from;
            same = t == p->plan_ids[i];
        }
        carried = same && patch_plan(p->views.data(), n, p->cow_copies == p->plan_copies_then, ph);
    }
    int rc = carried ? APAR_OK : build_plan(p->views.data(), n, p->ref.data(), p->seg_of.data(), prm, ph);
    if (rc != APAR_OK) {
        ph.reusable = false;
        return rc;
    }
    p->plan_ids.assign(ids, ids + n);
    p->plan_prm = prm;
    p->plan_threads_then = p->threads.size();
    p->plan_copies_then = p->cow_copies;
    (carried ? p->n_plans_carried : p->n_plans_built) += 1;
    const int64_t e = p->shape.dtype == APAR_F32 ? 4 : 2;
    apar_plan_info info{};
    info.n_threads = n;
    info.n_segments = ph.n_segments;
    info.n_units = (int64_t)ph.wgs.size() * p->shape.n_kv;
    info.n_partial_rows = ph.n_partial_rows;
    info.unique_blocks = ph.unique_blocks;
    info.unique_tokens = ph.unique_tokens;
    info.path_tokens = ph.path_tokens;
    info.algorithmic_bytes = ph.unique_tokens * 2 * p->shape.n_kv * p->shape.d * e +
                             2 * (int64_t)n * n_cand * p->shape.n_q * p->shape.d * e;
    if (p->shape.fp8_sealed)  // full blocks: one byte per element and two scales per (block, kv head)
        info.algorithmic_bytes -= ph.full_blocks * ((int64_t)kBlockTokens * p->shape.n_kv * p->shape.d * 2 - 8 * p->shape.n_kv);
    if (spec) info.algorithmic_bytes += 2 * (int64_t)n * n_cand * p->shape.n_kv * p->shape.d * e;
    p->plan_geom[0] = prm.rows_per_thread;
    p->plan_geom[2] = (prm.rows_per_thread + 15) / 16;
    p->plan_geom[1] = (prm.rows_per_thread + p->plan_geom[2] - 1) / p->plan_geom[2];
    if (p->dry_run) {
        p->last_plan = info;
        return APAR_OK;
    }
    DeviceGuard guard(p->device);
    hipStream_t st = (hipStream_t)stream;

    // stage the five tables in one copy
    size_t ofs[6];
    ofs[0] = 0;
    ofs[1] = align_up(ofs[0] + ph.wgs.size() * sizeof(WgDesc), 256);
    ofs[2] = align_up(ofs[1] + ph.tiles.size() * sizeof(TileRef), 256);
    ofs[3] = align_up(ofs[2] + ph.dfs_threads.size() * 4, 256);
    ofs[4] = align_up(ofs[3] + ph.path_ofs.size() * 4, 256);
    ofs[5] = align_up(ofs[4] + ph.path_ids.size() * 4, 256);
    const size_t slots = (size_t)ph.n_partial_rows * n_cand * p->shape.n_q;
    StageSlot* s = nullptr;
    char *host = nullptr, *dev = nullptr;
    PartialBuf part = p->part;
    if (p->resident_behind) p->resident = nullptr;
    p->resident_behind = false;
    // a carried-over plan whose tables are still on the device from the previous call: only the words that
    // changed are sent, and written in place once the previous call's kernels are through
    // (small tables are staged whole instead: one copy, against a copy and a launch)
    const bool in_place = carried && !fixed && p->resident && p->resident_bytes == ofs[5] && ofs[5] >= kCopyStreamMinBytes;
    if (!in_place) p->resident = nullptr;
    if (in_place) {
        p->resident_behind = true;
        StageSlot* res = p->resident;
        const size_t n_pairs = ph.dirty_wg_words.size() + ph.dirty_tile_words.size();
        if (n_pairs > 0) {
            StageSlot* ps = nullptr;
            if ((rc = acquire_stage(p, n_pairs * 2 * sizeof(int32_t), &ps)) != APAR_OK) return rc;
            int32_t* pairs = (int32_t*)ps->host;
            const int32_t* wg_words = (const int32_t*)ph.wgs.data();
            const int32_t* tile_words = (const int32_t*)ph.tiles.data();
            const int32_t wg_base = (int32_t)(ofs[0] / 4), tile_base = (int32_t)(ofs[1] / 4);
            for (int32_t w : ph.dirty_wg_words) *pairs++ = wg_base + w, *pairs++ = wg_words[w];
            for (int32_t w : ph.dirty_tile_words) *pairs++ = tile_base + w, *pairs++ = tile_words[w];
            if ((rc = upload(p, ps, n_pairs * 2 * sizeof(int32_t), st)) != APAR_OK) return rc;
            if (res->pending) HIP_TRY(hipStreamWaitEvent(st, res->ev, 0));  // (a no-op on the stream of the previous call)
            HIP_TRY(launch_scatter_words((int32_t*)res->dev, (const int32_t*)ps->dev, (int)n_pairs, st));
            HIP_TRY(hipEventRecord(ps->ev, st));
            ps->pending = true;
        }
        p->resident_behind = false;
        s = res;
        dev = res->dev;
    } else if (fixed) {
        // the workspace has a fixed size: a plan or a set of partial results beyond it is refused
        const size_t slot_bytes = (size_t)(p->shape.d + 2) * sizeof(float);
        const size_t cap_slots = kFixedPartBytes / slot_bytes;
        if (ofs[5] > kFixedPlanBytes || slots > cap_slots) return APAR_ERR_WORKSPACE_LIMIT;
        if (p->fixed_pending) {  // the previous call's upload may still be reading the pinned buffer
            HIP_TRY(hipEventSynchronize(p->fixed_up));
            p->fixed_pending = false;
        }
        host = p->fixed_host;
        dev = p->fixed_dev;
        part.o = (float*)(p->fixed_dev + kFixedPlanBytes);
        part.ml = part.o + cap_slots * p->shape.d;
    } else {
        if ((rc = acquire_stage(p, ofs[5], &s)) != APAR_OK) return rc;
        host = s->host;
        dev = s->dev;
    }
    if (!in_place) {
        memcpy(host + ofs[0], ph.wgs.data(), ph.wgs.size() * sizeof(WgDesc));
        memcpy(host + ofs[1], ph.tiles.data(), ph.tiles.size() * sizeof(TileRef));
        memcpy(host + ofs[2], ph.dfs_threads.data(), ph.dfs_threads.size() * 4);
        memcpy(host + ofs[3], ph.path_ofs.data(), ph.path_ofs.size() * 4);
        if (!ph.path_ids.empty()) memcpy(host + ofs[4], ph.path_ids.data(), ph.path_ids.size() * 4);
    }

    // partial-result buffer
    if (!fixed && slots > p->part_slots_cap) {
        HIP_TRY(hipDeviceSynchronize());
        if (p->part.o) HIP_TRY(hipFree(p->part.o));
        if (p->part.ml) HIP_TRY(hipFree(p->part.ml));
        p->part = PartialBuf{};
        p->part_slots_cap = 0;
        const size_t cap = slots + slots / 4 + 1024;
        HIP_TRY(hipMalloc((void**)&p->part.o, cap * p->shape.d * sizeof(float)));
        HIP_TRY(hipMalloc((void**)&p->part.ml, cap * 2 * sizeof(float)));
        p->part_slots_cap = cap;
        part = p->part;
    }

    if (in_place) {
        // (already there)
    } else if (fixed) {
        HIP_TRY(hipMemcpyAsync(dev, host, ofs[5], hipMemcpyHostToDevice, st));
        HIP_TRY(hipEventRecord(p->fixed_up, st));
        p->fixed_pending = true;
    } else if ((rc = upload(p, s, ofs[5], st)) != APAR_OK) {
        return rc;
    }
    PlanDev pd;
    pd.wgs = (const WgDesc*)(dev + ofs[0]);
    pd.tiles = (const TileRef*)(dev + ofs[1]);
    pd.dfs_threads = (const int32_t*)(dev + ofs[2]);
    pd.path_ofs = (const int32_t*)(dev + ofs[3]);
    pd.path_ids = (const int32_t*)(dev + ofs[4]);
    pd.n_wg = (int32_t)ph.wgs.size();
    for (int k = 0; k < 3; ++k) pd.n_wg_class[k] = ph.n_wg_class[k];
    if (pd.n_wg_class[0] + pd.n_wg_class[1] + pd.n_wg_class[2] != pd.n_wg) return APAR_ERR_INVALID_ARG;
    pd.n_threads = n;
    pd.rows_per_thread = p->plan_geom[0];
    pd.rows_per_slice = p->plan_geom[1];
    pd.n_slices = p->plan_geom[2];

    EventPair ev;
    const bool profiling = p->profiling && !fixed;
    if (profiling) {
        if ((rc = new_event(p, &ev.a)) != APAR_OK || (rc = new_event(p, &ev.b)) != APAR_OK ||
            (rc = new_event(p, &ev.c)) != APAR_OK)
            return rc;
        HIP_TRY(hipEventRecord(ev.a, st));
    }
    ClassStreams one_stream;
    one_stream.serial = true;
    HIP_TRY(launch_attention_partial(p->shape, p->kv, q, pd, n_cand, part, cand_k, cand_v, mask, out,
                                     fixed ? one_stream : p->class_streams, st));
    if (profiling) HIP_TRY(hipEventRecord(ev.b, st));
    if (ph.any_partial)
        HIP_TRY(launch_merge(p->shape, pd, part, q, cand_k, cand_v, mask, n_cand, out, st));
    if (profiling) {
        HIP_TRY(hipEventRecord(ev.c, st));
        p->decode_events.push_back(ev);
        p->n_decode_calls += 1;
    }
    if (s) {
        HIP_TRY(hipEventRecord(s->ev, st));
        s->pending = true;
        p->resident = s;
        p->resident_bytes = ofs[5];
    }
    p->last_plan = info;
    if (profiling)
        p->plan_host_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count() -
                           p->wait_in_call_ms;
    return APAR_OK;
}

// Mean attended rows per query token from which a bf16 prefill call goes to the 32x32 kernel by itself.
constexpr int64_t kMatrixPrefillMeanWalk = 1024;

// bf16 pools: the matrix-core prefill kernel.  One workgroup per (thread, chunk of 128 / group query tokens);
// the threads' block tables are staged next to the workgroup descriptors.
int prefill_bf16(apar_pool* p, const std::vector<PrefillThreadView>& views, int64_t rows, int64_t attended,
                 const void* q, void* out, void* stream, std::chrono::steady_clock::time_point t0) {
    const int group = p->shape.group;
    if (group < 1 || group > 16 || 16 % group != 0) return APAR_ERR_UNSUPPORTED;
    const int chunk = 128 / group;
    std::vector<PrefillWg>& wgs = p->prefill_wgs;
    std::vector<int32_t>& tables = p->prefill_tables;
    wgs.clear();
    tables.clear();
    for (const PrefillThreadView& t : views) {
        if (t.len > INT32_MAX / 2 || tables.size() + (size_t)t.n_blocks > (size_t)INT32_MAX / 2) return APAR_ERR_UNSUPPORTED;
        const int32_t table_ofs = (int32_t)tables.size();
        tables.insert(tables.end(), t.table, t.table + t.n_blocks);
        for (int64_t r0 = 0; r0 < t.m; r0 += chunk) {
            PrefillWg w{};
            w.table_ofs = table_ofs;
            w.q_row0 = (int32_t)(t.q_base + r0);
            w.p0 = (int32_t)(t.len - t.m + r0);
            w.n_tok = (int32_t)std::min<int64_t>(chunk, t.m - r0);
            w.len = (int32_t)t.len;
            wgs.push_back(w);
        }
    }
    // Workgroups of one tree (same first block) stay together, in the caller's order, so that the threads of a
    // tree walk their common prefix at about the same time and find it in the L2 of the XCD that serves their
    // kv head; trees with the longest walk go first so that the launch does not end on a long one.
    {
        std::unordered_map<int32_t, int32_t> longest;  // first block of a tree -> its longest walk
        for (const PrefillWg& w : wgs) {
            int32_t& e = longest[tables[w.table_ofs]];
            e = std::max(e, w.p0 + w.n_tok);
        }
        std::vector<std::pair<uint64_t, PrefillWg>> keyed;
        keyed.reserve(wgs.size());
        for (const PrefillWg& w : wgs) {
            const int32_t root = tables[w.table_ofs];
            keyed.emplace_back(((uint64_t)(uint32_t)(INT32_MAX - longest[root]) << 32) | (uint32_t)root, w);
        }
        std::stable_sort(keyed.begin(), keyed.end(),
                         [](const std::pair<uint64_t, PrefillWg>& a, const std::pair<uint64_t, PrefillWg>& b) {
                             return a.first < b.first;
                         });
        for (size_t i = 0; i < wgs.size(); ++i) wgs[i] = keyed[i].second;
    }
    apar_plan_info info{};
    info.n_threads = (int64_t)views.size();
    info.n_units = (int64_t)wgs.size() * p->shape.n_kv;
    info.path_tokens = attended;
    info.algorithmic_bytes = 2 * rows * p->shape.n_q * p->shape.d * 2;
    p->last_plan = info;
    DeviceGuard guard(p->device);
    hipStream_t st = (hipStream_t)stream;
    const size_t wg_bytes = align_up(wgs.size() * sizeof(PrefillWg), 256);
    const size_t table_bytes = tables.size() * sizeof(int32_t);
    StageSlot* s = nullptr;
    int rc = acquire_stage(p, wg_bytes + table_bytes, &s);
    if (rc != APAR_OK) return rc;
    memcpy(s->host, wgs.data(), wgs.size() * sizeof(PrefillWg));
    memcpy(s->host + wg_bytes, tables.data(), table_bytes);
    if ((rc = upload(p, s, wg_bytes + table_bytes, st)) != APAR_OK) return rc;
    EventPair ev;
    if (p->profiling) {
        if ((rc = new_event(p, &ev.a)) != APAR_OK || (rc = new_event(p, &ev.b)) != APAR_OK ||
            (rc = new_event(p, &ev.c)) != APAR_OK)
            return rc;
        HIP_TRY(hipEventRecord(ev.a, st));
    }
    HIP_TRY(launch_prefill_bf16(p->shape, p->kv, q, (const PrefillWg*)s->dev, (const int32_t*)(s->dev + wg_bytes),
                                (int)wgs.size(), out, st));
    if (p->profiling) {
        HIP_TRY(hipEventRecord(ev.b, st));
        HIP_TRY(hipEventRecord(ev.c, st));
        p->decode_events.push_back(ev);
        p->n_decode_calls += 1;
    }
    HIP_TRY(hipEventRecord(s->ev, st));
    s->pending = true;
    if (p->profiling)
        p->plan_host_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count() -
                           p->wait_in_call_ms;
    return APAR_OK;
}

int prefill_common(apar_pool* p, const void* q, const apar_thread* ids, const int32_t* m, int n, void* out,
                   void* stream) {
    if (!p || n < 0) return APAR_ERR_INVALID_ARG;
    if (n == 0) return APAR_OK;
    if (!ids || !m) return APAR_ERR_INVALID_ARG;
    if (p->dry_run ? (q || out) : (!q || !out)) return APAR_ERR_INVALID_ARG;
    const auto t0 = std::chrono::steady_clock::now();
    p->wait_in_call_ms = 0.0;
    std::vector<PrefillThreadView>& views = p->prefill_views;
    views.resize(n);
    int64_t rows = 0, attended = 0;
    for (int i = 0; i < n; ++i) {
        Thread* t = live_thread(p, ids[i]);
        if (!t) return APAR_ERR_INVALID_THREAD;
        if (m[i] < 1 || m[i] > t->len) return APAR_ERR_INVALID_ARG;
        views[i] = PrefillThreadView{t->table.data(), (int32_t)t->table.size(), t->len, m[i], rows};
        rows += m[i];
        attended += (int64_t)m[i] * (t->len - m[i]) + (int64_t)m[i] * (m[i] + 1) / 2;
    }
    if (rows > INT32_MAX / 2) return APAR_ERR_UNSUPPORTED;
    PlanHost& ph = p->plan;
    int rc = APAR_OK;
    // bf16 pools have two kernels.  The 32x32 matrix-core kernel pays off once the walk of a query token is long
    // (its fixed cost per workgroup is spread over many super-blocks); short walks stay on the row-tile kernel,
    // whose plan also reads a prefix shared by sibling threads once for all of them.
    p->last_prefill_kernel = APAR_PREFILL_ROW_TILES;
    if (!p->dry_run && p->shape.dtype == APAR_BF16 && !p->shape.fp8_sealed && 16 % p->shape.group == 0 &&
        (p->prefill_kernel == APAR_PREFILL_MATRIX ||
         (p->prefill_kernel == APAR_PREFILL_AUTO && attended >= kMatrixPrefillMeanWalk * rows))) {
        p->last_prefill_kernel = APAR_PREFILL_MATRIX;
        return prefill_bf16(p, views, rows, attended, q, out, stream, t0);
    }
    rc = build_prefill_plan(views.data(), n, p->shape.group, ph);
    if (rc != APAR_OK) return rc;
    apar_plan_info info{};
    info.n_threads = n;
    info.n_units = (int64_t)ph.wgs.size() * p->shape.n_kv;
    info.path_tokens = attended;  // (query token, attended row) pairs
    const int64_t e = p->shape.dtype == APAR_F32 ? 4 : 2;
    info.algorithmic_bytes = 2 * rows * p->shape.n_q * p->shape.d * e;  // queries in, outputs out; K,V reads depend on caching
    p->plan_geom[0] = p->plan_geom[1] = p->shape.group;
    p->plan_geom[2] = 1;
    p->last_plan = info;
    if (p->dry_run) return APAR_OK;
    DeviceGuard guard(p->device);
    hipStream_t st = (hipStream_t)stream;
    const size_t wg_bytes = align_up(ph.wgs.size() * sizeof(WgDesc), 256);
    const size_t tile_bytes = ph.tiles.size() * sizeof(TileRef);
    StageSlot* s = nullptr;
    if ((rc = acquire_stage(p, wg_bytes + tile_bytes, &s)) != APAR_OK) return rc;
    memcpy(s->host, ph.wgs.data(), ph.wgs.size() * sizeof(WgDesc));
    if (tile_bytes) memcpy(s->host + wg_bytes, ph.tiles.data(), tile_bytes);
    if ((rc = upload(p, s, wg_bytes + tile_bytes, st)) != APAR_OK) return rc;
    PlanDev pd{};
    pd.wgs = (const WgDesc*)s->dev;
    pd.tiles = (const TileRef*)(s->dev + wg_bytes);
    pd.dfs_threads = nullptr;  // a row group is a query token, numbered as q_dev's rows are
    pd.path_ofs = pd.path_ids = nullptr;
    pd.n_wg = (int32_t)ph.wgs.size();
    for (int k = 0; k < 3; ++k) pd.n_wg_class[k] = ph.n_wg_class[k];
    pd.n_threads = (int32_t)rows;
    pd.rows_per_thread = pd.rows_per_slice = p->shape.group;
    pd.n_slices = 1;
    EventPair ev;
    if (p->profiling) {
        if ((rc = new_event(p, &ev.a)) != APAR_OK || (rc = new_event(p, &ev.b)) != APAR_OK ||
            (rc = new_event(p, &ev.c)) != APAR_OK)
            return rc;
        HIP_TRY(hipEventRecord(ev.a, st));
    }
    HIP_TRY(launch_attention_partial(p->shape, p->kv, q, pd, 1, p->part, nullptr, nullptr, nullptr, out,
                                     p->class_streams, st));
    if (p->profiling) {
        HIP_TRY(hipEventRecord(ev.b, st));
        HIP_TRY(hipEventRecord(ev.c, st));
        p->decode_events.push_back(ev);
        p->n_decode_calls += 1;
    }
    HIP_TRY(hipEventRecord(s->ev, st));
    s->pending = true;
    if (p->profiling)
        p->plan_host_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count() -
                           p->wait_in_call_ms;
    return APAR_OK;
}

}  // namespace

// ===========================================================================
// C ABI
// ===========================================================================
extern "C" {

int apar_pool_create(const apar_pool_config* cfg, void* kv_dev, size_t kv_bytes, apar_pool** out) {
    if (!cfg || !out) return APAR_ERR_INVALID_ARG;
    if (!kv_dev && kv_bytes != 0) return APAR_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->block_size != kBlockTokens) return APAR_ERR_INVALID_ARG;
    if (cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return APAR_ERR_INVALID_ARG;
    if (cfg->num_blocks < 1 || cfg->num_blocks > kMaxPoolBlocks || cfg->max_threads < 1)
        return APAR_ERR_INVALID_ARG;
    if (cfg->dtype != APAR_F32 && cfg->dtype != APAR_BF16 && cfg->dtype != APAR_BF16_FP8KV) return APAR_ERR_INVALID_ARG;
    if (!(cfg->softmax_scale >= 0.0f) || !std::isfinite(cfg->softmax_scale)) return APAR_ERR_INVALID_ARG;
    if (cfg->dtype != APAR_F32 && cfg->head_dim != 128) return APAR_ERR_UNSUPPORTED;
    if (cfg->dtype == APAR_F32 && cfg->head_dim != 64 && cfg->head_dim != 128) return APAR_ERR_UNSUPPORTED;
    if (cfg->n_q_heads / cfg->n_kv_heads > 16) return APAR_ERR_UNSUPPORTED;
    const int64_t e = cfg->dtype == APAR_F32 ? 4 : 2;
    const int64_t tile = 2 * (int64_t)kBlockTokens * cfg->head_dim * e;
    const int64_t block = tile * cfg->n_kv_heads;
    if (kv_dev && ((uint64_t)kv_bytes < (uint64_t)(block * cfg->num_blocks) || ((uintptr_t)kv_dev & 255)))
        return APAR_ERR_INVALID_ARG;

    apar_pool* p = new (std::nothrow) apar_pool();
    if (!p) return APAR_ERR_INVALID_ARG;
    p->cfg = *cfg;
    p->kv = (char*)kv_dev;
    p->dry_run = kv_dev == nullptr;
    if (!p->dry_run) {
        if (!hip_ok(hipGetDevice(&p->device), "hipGetDevice")) {
            delete p;
            return APAR_ERR_HIP;
        }
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, kv_dev) == hipSuccess) p->device = attr.device;
        else (void)hipGetLastError();
        // what apar_decode_attention_fixed needs and may not obtain itself: the address of this device's copy of
        // the static workspace, a pinned buffer to stage its plan in and the event that follows the upload
        DeviceGuard guard(p->device);
        int rc = APAR_OK;
        if (!hip_ok(fixed_workspace_of_device(p->device, &p->fixed_dev), "hipGetSymbolAddress(scratch)")) rc = APAR_ERR_HIP;
        if (rc == APAR_OK && !hip_ok(hipHostMalloc((void**)&p->fixed_host, kFixedPlanBytes, hipHostMallocDefault), "hipHostMalloc"))
            rc = APAR_ERR_HIP;
        if (rc == APAR_OK && !hip_ok(hipEventCreateWithFlags(&p->fixed_up, hipEventDisableTiming), "hipEventCreate"))
            rc = APAR_ERR_HIP;
        if (rc != APAR_OK) {
            if (p->fixed_host) (void)hipHostFree(p->fixed_host);
            delete p;
            return rc;
        }
    }
    const float scale = cfg->softmax_scale > 0.0f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
    p->shape.n_q = cfg->n_q_heads;
    p->shape.n_kv = cfg->n_kv_heads;
    p->shape.d = cfg->head_dim;
    p->shape.group = cfg->n_q_heads / cfg->n_kv_heads;
    p->shape.dtype = cfg->dtype == APAR_F32 ? APAR_F32 : APAR_BF16;
    p->shape.fp8_sealed = cfg->dtype == APAR_BF16_FP8KV ? 1 : 0;
    p->shape.scale_log2e = scale * 1.4426950408889634f;
    p->shape.tile_bytes = tile;
    p->shape.block_bytes = block;
    p->ref.assign(cfg->num_blocks, 0);
    p->free_stack.resize(cfg->num_blocks);
    for (int64_t i = 0; i < cfg->num_blocks; ++i) p->free_stack[i] = (int32_t)(cfg->num_blocks - 1 - i);
    p->seg_of.assign(cfg->num_blocks, -1);
    *out = p;
    return APAR_OK;
}

int apar_pool_destroy(apar_pool* p) {
    if (!p) return APAR_OK;
    if (p->dry_run) {
        delete p;
        return APAR_OK;
    }
    DeviceGuard guard(p->device);
    int rc = APAR_OK;
    if (!hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize")) rc = APAR_ERR_HIP;
    for (StageSlot& s : p->stage) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.dev) (void)hipFree(s.dev);
        if (s.ev) (void)hipEventDestroy(s.ev);
        if (s.up) (void)hipEventDestroy(s.up);
    }
    if (p->copy_stream) (void)hipStreamDestroy(p->copy_stream);
    if (p->fixed_host) (void)hipHostFree(p->fixed_host);
    if (p->fixed_up) (void)hipEventDestroy(p->fixed_up);
    if (p->part.o) (void)hipFree(p->part.o);
    if (p->part.ml) (void)hipFree(p->part.ml);
    auto drop = [](hipEvent_t e) {
        if (e) (void)hipEventDestroy(e);
    };
    for (EventPair& e : p->decode_events) drop(e.a), drop(e.b), drop(e.c);
    for (EventPair& e : p->append_events) drop(e.a), drop(e.b), drop(e.c);
    for (hipEvent_t e : p->spare_events) drop(e);
    drop(p->class_streams.fork), drop(p->class_streams.join[0]), drop(p->class_streams.join[1]);
    for (hipStream_t a : p->class_streams.aux)
        if (a) (void)hipStreamDestroy(a);
    delete p;
    return rc;
}

int apar_thread_create(apar_pool* p, apar_thread* out) {
    if (!p || !out) return APAR_ERR_INVALID_ARG;
    if ((int64_t)p->threads.size() >= p->cfg.max_threads) return APAR_ERR_THREAD_CAPACITY;
    p->threads.emplace_back();
    p->threads.back().live = true;
    p->live_threads += 1;
    *out = (apar_thread)(p->threads.size() - 1);
    return APAR_OK;
}

int apar_fork(apar_pool* p, apar_thread parent, int n_children, apar_thread* children_out) {
    if (!p || !children_out) return APAR_ERR_INVALID_ARG;
    if (!live_thread(p, parent)) return APAR_ERR_INVALID_THREAD;
    if (n_children < 1) return APAR_ERR_INVALID_ARG;
    if ((int64_t)p->threads.size() + n_children > p->cfg.max_threads) return APAR_ERR_THREAD_CAPACITY;
    // (no exact-size reserve here: it would re-allocate the whole thread array on every fork)
    for (int c = 0; c < n_children; ++c) {
        p->threads.emplace_back();
        Thread& child = p->threads.back();
        const Thread& par = p->threads[parent];
        child.live = true;
        child.len = par.len;
        child.forked_from = parent;
        child.table = par.table;
        children_out[c] = (apar_thread)(p->threads.size() - 1);
    }
    for (int32_t b : p->threads[parent].table) p->ref[b] += n_children;
    p->live_threads += n_children;
    return APAR_OK;
}

int apar_append_kv(apar_pool* p, apar_thread thread, const void* k_dev, const void* v_dev, int n_tokens,
                   void* hip_stream) {
    if (!p || n_tokens < 0) return APAR_ERR_INVALID_ARG;
    Thread* t = live_thread(p, thread);
    if (!t) return APAR_ERR_INVALID_THREAD;
    if (n_tokens == 0) return APAR_OK;
    if (p->dry_run ? (k_dev || v_dev) : (!k_dev || !v_dev)) return APAR_ERR_INVALID_ARG;
    const int64_t B = kBlockTokens;
    int64_t need = (t->len + n_tokens + B - 1) / B - (t->len + B - 1) / B;
    if (t->len % B != 0 && p->ref[t->table.back()] > 1) need += 1;
    if (need > (int64_t)p->free_stack.size()) return APAR_ERR_OUT_OF_BLOCKS;
    std::vector<int32_t> codes(n_tokens), copies, seals;
    for (int i = 0; i < n_tokens; ++i) codes[i] = append_one(p, *t, copies, seals);
    if (p->check_writes && writes_are_private(p, codes, copies, seals) != APAR_OK) return APAR_ERR_INTERNAL;
    if (p->dry_run) return APAR_OK;
    DeviceGuard guard(p->device);
    return run_append(p, codes, copies, seals, nullptr, k_dev, v_dev, (hipStream_t)hip_stream);
}

// One row per entry of `threads` (a thread may repeat), row i taken from row src_rows[i] of k_dev, v_dev
// (row i if src_rows is null).  All or nothing.
static int append_rows_of(apar_pool* p, const apar_thread* threads, int n, const std::vector<int32_t>* src_rows,
                          const void* k_dev, const void* v_dev, void* hip_stream) {
    if ((int64_t)p->free_stack.size() < n) {
        // Each row takes at most one block, so only a nearly full pool needs the
        // exact count: replay the policy on scratch copies of what it reads.
        struct Sim {
            int64_t len;
            bool private_tail;  // an earlier row of this call already made the tail this thread's own
        };
        std::unordered_map<int32_t, Sim> sim;         // by thread id
        std::unordered_map<int32_t, int32_t> dropped;  // references copy-on-write took off a block so far
        int64_t need = 0;
        for (int i = 0; i < n; ++i) {
            const Thread& t = p->threads[threads[i]];
            auto it = sim.find(threads[i]);
            if (it == sim.end()) it = sim.emplace(threads[i], Sim{t.len, false}).first;
            Sim& s = it->second;
            if (s.len % kBlockTokens == 0) {
                need += 1;
                s.private_tail = true;
            } else if (!s.private_tail) {
                const int32_t tail = t.table.back();
                int32_t& d = dropped[tail];
                if (p->ref[tail] - d > 1) {
                    need += 1;
                    d += 1;
                    s.private_tail = true;
                }
            }
            s.len += 1;
        }
        if (need > (int64_t)p->free_stack.size()) return APAR_ERR_OUT_OF_BLOCKS;
    }
    std::vector<int32_t>& codes = p->scratch_codes;
    std::vector<int32_t>& copies = p->scratch_copies;
    std::vector<int32_t>& seals = p->scratch_seals;
    codes.resize(n);
    copies.clear();
    seals.clear();
    for (int i = 0; i < n; ++i) codes[i] = append_one(p, p->threads[threads[i]], copies, seals);
    if (p->check_writes && writes_are_private(p, codes, copies, seals) != APAR_OK) return APAR_ERR_INTERNAL;
    if (p->dry_run) return APAR_OK;
    DeviceGuard guard(p->device);
    return run_append(p, codes, copies, seals, src_rows, k_dev, v_dev, (hipStream_t)hip_stream);
}

int apar_append_kv_batch(apar_pool* p, const apar_thread* threads, int n, const void* k_dev, const void* v_dev,
                         void* hip_stream) {
    if (!p || n < 0) return APAR_ERR_INVALID_ARG;
    if (n == 0) return APAR_OK;
    if (!threads) return APAR_ERR_INVALID_ARG;
    if (p->dry_run ? (k_dev || v_dev) : (!k_dev || !v_dev)) return APAR_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (!live_thread(p, threads[i])) return APAR_ERR_INVALID_THREAD;
    return append_rows_of(p, threads, n, nullptr, k_dev, v_dev, hip_stream);
}

int apar_append_kv_gather(apar_pool* p, const apar_thread* threads, const int32_t* src_rows, int n, const void* k_dev,
                          const void* v_dev, void* hip_stream) {
    if (!p || n < 0) return APAR_ERR_INVALID_ARG;
    if (n == 0) return APAR_OK;
    if (!threads || !src_rows) return APAR_ERR_INVALID_ARG;
    if (p->dry_run ? (k_dev || v_dev) : (!k_dev || !v_dev)) return APAR_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i) {
        if (!live_thread(p, threads[i])) return APAR_ERR_INVALID_THREAD;
        if (src_rows[i] < 0) return APAR_ERR_INVALID_ARG;
    }
    std::vector<int32_t>& src = p->scratch_commit_src;
    src.assign(src_rows, src_rows + n);
    return append_rows_of(p, threads, n, &src, k_dev, v_dev, hip_stream);
}

int apar_commit_candidates(apar_pool* p, const apar_thread* threads, int n, const void* cand_k_dev,
                           const void* cand_v_dev, int n_cand, const uint8_t* accept_masks, void* hip_stream) {
    if (!p || n < 0 || n_cand < 1 || n_cand > 8) return APAR_ERR_INVALID_ARG;
    if (n == 0) return APAR_OK;
    if (!threads || !accept_masks) return APAR_ERR_INVALID_ARG;
    if (p->dry_run ? (cand_k_dev || cand_v_dev) : (!cand_k_dev || !cand_v_dev)) return APAR_ERR_INVALID_ARG;
    if ((int64_t)n * n_cand > INT32_MAX) return APAR_ERR_INVALID_ARG;
    std::vector<apar_thread>& ids = p->scratch_commit_ids;
    std::vector<int32_t>& src = p->scratch_commit_src;
    ids.clear();
    src.clear();
    for (int i = 0; i < n; ++i) {
        if (!live_thread(p, threads[i])) return APAR_ERR_INVALID_THREAD;
        const uint32_t bits = accept_masks[i];
        if (bits >> n_cand) return APAR_ERR_INVALID_ARG;  // a candidate that does not exist
        for (int c = 0; c < n_cand; ++c)
            if ((bits >> c) & 1u) {
                ids.push_back(threads[i]);
                src.push_back(i * n_cand + c);
            }
    }
    if (ids.empty()) return APAR_OK;
    return append_rows_of(p, ids.data(), (int)ids.size(), &src, cand_k_dev, cand_v_dev, hip_stream);
}

int apar_decode_attention(apar_pool* p, const void* q_dev, const apar_thread* threads, int n, void* out_dev,
                          void* hip_stream) {
    return decode_common(p, q_dev, nullptr, nullptr, nullptr, 1, threads, n, out_dev, hip_stream, false);
}

int apar_decode_attention_spec(apar_pool* p, const void* q_dev, const void* cand_k_dev, const void* cand_v_dev,
                               const uint8_t* mask_dev, int n_cand, const apar_thread* threads, int n, void* out_dev,
                               void* hip_stream) {
    return decode_common(p, q_dev, cand_k_dev, cand_v_dev, mask_dev, n_cand, threads, n, out_dev, hip_stream, true);
}

int apar_decode_attention_fixed(apar_pool* p, const void* q_dev, const apar_thread* threads, int n, void* out_dev,
                                void* hip_stream) {
    return decode_common(p, q_dev, nullptr, nullptr, nullptr, 1, threads, n, out_dev, hip_stream, false, true);
}

int apar_prefill_attention(apar_pool* p, const void* q_dev, const apar_thread* threads, const int32_t* m, int n,
                           void* out_dev, void* hip_stream) {
    return prefill_common(p, q_dev, threads, m, n, out_dev, hip_stream);
}

int apar_free_thread(apar_pool* p, apar_thread thread) {
    if (!p) return APAR_ERR_INVALID_ARG;
    Thread* t = live_thread(p, thread);
    if (!t) return APAR_ERR_INVALID_THREAD;
    for (size_t i = t->table.size(); i-- > 0;) {
        const int32_t b = t->table[i];
        if (--p->ref[b] == 0) p->free_stack.push_back(b);
    }
    t->live = false;
    t->len = 0;
    std::vector<int32_t>().swap(t->table);
    p->live_threads -= 1;
    return APAR_OK;
}

int apar_thread_len(apar_pool* p, apar_thread thread, int64_t* len_out) {
    if (!p || !len_out) return APAR_ERR_INVALID_ARG;
    Thread* t = live_thread(p, thread);
    if (!t) return APAR_ERR_INVALID_THREAD;
    *len_out = t->len;
    return APAR_OK;
}

int apar_thread_block_table(apar_pool* p, apar_thread thread, int32_t* table_out, int cap, int* n_out) {
    if (!p || !n_out || cap < 0 || (cap > 0 && !table_out)) return APAR_ERR_INVALID_ARG;
    Thread* t = live_thread(p, thread);
    if (!t) return APAR_ERR_INVALID_THREAD;
    *n_out = (int)t->table.size();
    if ((size_t)cap < t->table.size()) return APAR_ERR_INVALID_ARG;
    if (!t->table.empty()) memcpy(table_out, t->table.data(), t->table.size() * sizeof(int32_t));
    return APAR_OK;
}

int apar_block_refcount(apar_pool* p, int32_t block, int32_t* refcount_out) {
    if (!p || !refcount_out || block < 0 || block >= p->cfg.num_blocks) return APAR_ERR_INVALID_ARG;
    *refcount_out = p->ref[block];
    return APAR_OK;
}

int apar_pool_stats(apar_pool* p, apar_stats* out) {
    if (!p || !out) return APAR_ERR_INVALID_ARG;
    out->total_blocks = p->cfg.num_blocks;
    out->free_blocks = (int64_t)p->free_stack.size();
    out->used_blocks = out->total_blocks - out->free_blocks;
    out->live_threads = p->live_threads;
    out->threads_issued = (int64_t)p->threads.size();
    out->cow_copies = p->cow_copies;
    out->block_bytes = p->shape.block_bytes;
    out->bytes_resident = out->used_blocks * p->shape.block_bytes;
    int64_t vanilla = 0;
    for (const Thread& t : p->threads)
        if (t.live) vanilla += (int64_t)t.table.size();
    out->bytes_vanilla = vanilla * p->shape.block_bytes;
    return APAR_OK;
}

int apar_last_plan_info(apar_pool* p, apar_plan_info* out) {
    if (!p || !out) return APAR_ERR_INVALID_ARG;
    *out = p->last_plan;
    return APAR_OK;
}

int apar_last_plan_export(apar_pool* p, int which, int32_t* out, int64_t cap, int64_t* n_out) {
    if (!p || !n_out || cap < 0 || (cap > 0 && !out)) return APAR_ERR_INVALID_ARG;
    const PlanHost& ph = p->plan;
    const int32_t* src = nullptr;
    int64_t n = 0;
    switch (which) {
        case APAR_PLAN_WORKGROUPS: src = (const int32_t*)ph.wgs.data(), n = (int64_t)ph.wgs.size() * 32; break;
        case APAR_PLAN_TILES: src = (const int32_t*)ph.tiles.data(), n = (int64_t)ph.tiles.size() * 2; break;
        case APAR_PLAN_DFS_THREADS: src = ph.dfs_threads.data(), n = (int64_t)ph.dfs_threads.size(); break;
        case APAR_PLAN_PATH_OFS: src = ph.path_ofs.data(), n = (int64_t)ph.path_ofs.size(); break;
        case APAR_PLAN_PATH_IDS: src = ph.path_ids.data(), n = (int64_t)ph.path_ids.size(); break;
        case APAR_PLAN_GEOMETRY: src = p->plan_geom, n = 3; break;
        case APAR_PLAN_CHANGED_WORKGROUP_WORDS: src = ph.dirty_wg_words.data(), n = (int64_t)ph.dirty_wg_words.size(); break;
        case APAR_PLAN_CHANGED_TILE_WORDS: src = ph.dirty_tile_words.data(), n = (int64_t)ph.dirty_tile_words.size(); break;
        default: return APAR_ERR_INVALID_ARG;
    }
    *n_out = n;
    if (cap < n) return APAR_ERR_INVALID_ARG;
    if (n > 0) memcpy(out, src, (size_t)n * sizeof(int32_t));
    return APAR_OK;
}

int apar_read_kv_rows(apar_pool* p, apar_thread thread, int64_t first, int n, void* k_out_dev, void* v_out_dev,
                      void* hip_stream) {
    if (!p || n < 0 || first < 0) return APAR_ERR_INVALID_ARG;
    Thread* t = live_thread(p, thread);
    if (!t) return APAR_ERR_INVALID_THREAD;
    if (first + n > t->len || p->dry_run) return APAR_ERR_INVALID_ARG;
    if (n == 0) return APAR_OK;
    if (!k_out_dev || !v_out_dev) return APAR_ERR_INVALID_ARG;
    DeviceGuard guard(p->device);
    hipStream_t st = (hipStream_t)hip_stream;
    StageSlot* s = nullptr;
    int rc = acquire_stage(p, (size_t)n * sizeof(int32_t), &s);
    if (rc != APAR_OK) return rc;
    int32_t* codes = (int32_t*)s->host;
    for (int i = 0; i < n; ++i) {
        const int64_t pos = first + i;
        const bool sealed = p->shape.dtype == APAR_BF16 && (pos / kBlockTokens + 1) * kBlockTokens <= t->len;
        codes[i] = slot_code(*t, pos) | (sealed ? kCodeSealed : 0);
    }
    if ((rc = upload(p, s, (size_t)n * sizeof(int32_t), st)) != APAR_OK) return rc;
    HIP_TRY(launch_read_rows(p->shape, p->kv, (const int32_t*)s->dev, n, k_out_dev, v_out_dev, st));
    HIP_TRY(hipEventRecord(s->ev, st));
    s->pending = true;
    return APAR_OK;
}

int apar_profile_enable(apar_pool* p, int on) {
    if (!p) return APAR_ERR_INVALID_ARG;
    p->profiling = on != 0;
    return APAR_OK;
}

int apar_profile_read(apar_pool* p, apar_profile* out) {
    if (!p || !out) return APAR_ERR_INVALID_ARG;
    memset(out, 0, sizeof(*out));
    p->last_attention_ms.clear();
    if (p->dry_run) return APAR_OK;
    DeviceGuard guard(p->device);
    for (EventPair& e : p->decode_events) {
        float ms = 0.0f;
        HIP_TRY(hipEventSynchronize(e.c));
        HIP_TRY(hipEventElapsedTime(&ms, e.a, e.b));
        out->attention_kernel_ms += ms;
        p->last_attention_ms.push_back(ms);
        HIP_TRY(hipEventElapsedTime(&ms, e.b, e.c));
        out->merge_kernel_ms += ms;
        p->spare_events.push_back(e.a);
        p->spare_events.push_back(e.b);
        p->spare_events.push_back(e.c);
    }
    for (EventPair& e : p->append_events) {
        float ms = 0.0f;
        HIP_TRY(hipEventSynchronize(e.b));
        HIP_TRY(hipEventElapsedTime(&ms, e.a, e.b));
        out->append_kernels_ms += ms;
        p->spare_events.push_back(e.a);
        p->spare_events.push_back(e.b);
    }
    out->n_decode_calls = p->n_decode_calls;
    out->n_append_calls = p->n_append_calls;
    out->plan_host_ms = p->plan_host_ms;
    out->host_wait_ms = p->host_wait_ms;
    p->decode_events.clear();
    p->append_events.clear();
    p->n_decode_calls = p->n_append_calls = 0;
    p->plan_host_ms = p->host_wait_ms = 0.0;
    return APAR_OK;
}

int apar_profile_attention_calls(apar_pool* p, float* ms_out, int64_t cap, int64_t* n_out) {
    if (!p || !n_out || cap < 0 || (cap > 0 && !ms_out)) return APAR_ERR_INVALID_ARG;
    const int64_t n = (int64_t)p->last_attention_ms.size();
    *n_out = n;
    if (cap < n) return APAR_ERR_INVALID_ARG;
    if (n > 0) memcpy(ms_out, p->last_attention_ms.data(), (size_t)n * sizeof(float));
    return APAR_OK;
}

int apar_plan_record_version(void) { return APAR_PLAN_RECORD_VERSION; }

int apar_set_plan_reuse(apar_pool* p, int on) {
    if (!p) return APAR_ERR_INVALID_ARG;
    p->plan_reuse = on != 0;
    return APAR_OK;
}

int apar_plan_counts(apar_pool* p, int64_t* n_built, int64_t* n_carried) {
    if (!p || !n_built || !n_carried) return APAR_ERR_INVALID_ARG;
    *n_built = p->n_plans_built;
    *n_carried = p->n_plans_carried;
    return APAR_OK;
}

int apar_set_write_checks(apar_pool* p, int on) {
    if (!p) return APAR_ERR_INVALID_ARG;
    p->check_writes = on != 0;
    return APAR_OK;
}

int apar_set_inline_shared(apar_pool* p, int on) {
    if (!p) return APAR_ERR_INVALID_ARG;
    p->inline_shared = on != 0;
    return APAR_OK;
}

int apar_set_matrix_units(apar_pool* p, int min_rows, int min_blocks) {
    if (!p || min_rows < 0 || min_blocks < 0) return APAR_ERR_INVALID_ARG;
    p->matrix_min_rows = min_rows;
    p->matrix_min_blocks = min_blocks;
    return APAR_OK;
}

int apar_set_prefill_kernel(apar_pool* p, int which) {
    if (!p || which < APAR_PREFILL_AUTO || which > APAR_PREFILL_MATRIX) return APAR_ERR_INVALID_ARG;
    p->prefill_kernel = which;
    return APAR_OK;
}

int apar_last_prefill_kernel(apar_pool* p) { return p ? p->last_prefill_kernel : 0; }

int apar_set_chunk_blocks(apar_pool* p, int blocks_per_unit) {
    if (!p || blocks_per_unit < 1 || blocks_per_unit > 65536) return APAR_ERR_INVALID_ARG;
    p->max_unit_tiles = blocks_per_unit;
    return APAR_OK;
}

const char* apar_status_string(int status) {
    switch (status) {
        case APAR_OK: return "ok";
        case APAR_ERR_INVALID_ARG: return "invalid argument";
        case APAR_ERR_INVALID_THREAD: return "invalid thread";
        case APAR_ERR_OUT_OF_BLOCKS: return "out of blocks";
        case APAR_ERR_THREAD_CAPACITY: return "thread capacity exceeded";
        case APAR_ERR_HIP: return "HIP runtime error";
        case APAR_ERR_UNSUPPORTED: return "unsupported shape";
        case APAR_ERR_WORKSPACE_LIMIT: return "call exceeds the fixed workspace";
        case APAR_ERR_INTERNAL: return "internal invariant violated";
        default: return "unknown status";
    }
}

const char* apar_last_hip_error(void) { return g_last_hip_error.c_str(); }

}  // extern "C"
