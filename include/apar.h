/*
 * apar.h - C ABI of the fork-tree paged-KV decode path of APAR
 * (auto-parallel auto-regressive decoding, arXiv 2401.06761) for AMD MI355X.
 *
 * The library keeps a fixed pool of 16-token KV blocks in caller-owned device
 * memory.  A generation thread (the paper's "sequence", Sec. 2.3) is a length
 * and a table of block ids.  A fork gives children the parent's table instead
 * of copies of its KV rows (Sec. 2.3: the fork shares the prefix and copies at
 * most one block), a finished thread gives back the blocks only it holds
 * (Alg. 1 ReleaseCache; Sec. 2.4 feature 2), and a decoding token attends to
 * the tokens on its own root path and to nothing else (Sec. 2.2 "Training
 * attention"; Sec. 2.4 feature 3).
 *
 * Conventions for every call
 *   - returns an apar_status; never throws, never aborts;
 *   - pointers named *_dev are DEVICE pointers, every other pointer is a HOST
 *     pointer.  The caller owns all of them, the KV pool buffer included, and
 *     must keep device buffers alive until the stream has run the work;
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Device work is enqueued on it and the call returns without
 *     waiting.  Host bookkeeping changes at call time, so introspection
 *     reflects every earlier call.  Calls on one pool must be issued from one
 *     host thread, and on one stream at a time (work on different streams
 *     must be ordered by the caller).  Parts of a call may run on streams
 *     that the pool owns (large table uploads, kernels of different classes
 *     side by side); they are ordered before and after `hip_stream` with
 *     events, so the caller sees the call as work on `hip_stream` alone, but
 *     a call may allocate staging memory and cannot be captured into a graph;
 *   - a call that fails with any status but APAR_ERR_HIP leaves the pool exactly
 *     as it was; after APAR_ERR_HIP the pool should be destroyed;
 *   - the layout of the pool buffer is private to the library (KV tiles are
 *     stored in the operand order of the matrix cores, not row-major).
 */
#ifndef APAR_H
#define APAR_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__) || defined(__clang__)
#define APAR_API __attribute__((visibility("default")))
#else
#define APAR_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct apar_pool apar_pool; /* opaque; created and destroyed by the library */
typedef int32_t apar_thread;        /* >= 0; issued 0, 1, 2, ... per pool; never reused */

typedef enum apar_status {
    APAR_OK = 0,
    APAR_ERR_INVALID_ARG = -1,     /* bad pointer, size, count or configuration          */
    APAR_ERR_INVALID_THREAD = -2,  /* id never issued, or already freed                  */
    APAR_ERR_OUT_OF_BLOCKS = -3,   /* the pool cannot supply the blocks the call needs   */
    APAR_ERR_THREAD_CAPACITY = -4, /* more than max_threads ids would be issued          */
    APAR_ERR_HIP = -5,             /* a HIP runtime call failed (see apar_last_hip_error) */
    APAR_ERR_UNSUPPORTED = -6,     /* shape outside what the kernels are built for       */
    APAR_ERR_WORKSPACE_LIMIT = -7, /* apar_decode_attention_fixed: the call needs more than */
                                   /* the fixed workspace holds; nothing was enqueued       */
    APAR_ERR_INTERNAL = -8         /* a write check (apar_set_write_checks) found a kernel  */
                                   /* about to write a block that other threads hold; nothing */
                                   /* was launched, the pool should be destroyed             */
} apar_status;

/* Pool types.  APAR_BF16_FP8KV: K, V, Q and the output are bf16 at the interface, as for APAR_BF16, but a
 * block whose sixteen slots are written is kept in fp8 (OCP e4m3, round to nearest even, saturating at 448)
 * with one power-of-two scale per (block, kv head) for K and one for V, chosen so that the largest magnitude
 * of the tile lands in the top binade of the format; a block that is still filling stays bf16.  Decode
 * attention then reads half the bytes per cached token (Sec. 3.3 measures throughput against the memory the
 * KV cache takes).  The kernels multiply the stored codes by the scale on their way into the bf16 matrix-core
 * operands, so the arithmetic is that of a bf16 pool holding the rounded values.  Blocks keep their bf16
 * size in the pool buffer (a block must be able to hold sixteen bf16 rows while it fills). */
enum { APAR_F32 = 0, APAR_BF16 = 1, APAR_BF16_FP8KV = 2 };

typedef struct apar_pool_config {
    int32_t n_q_heads;   /* Hq; multiple of n_kv_heads                                   */
    int32_t n_kv_heads;  /* Hkv                                                          */
    int32_t head_dim;    /* d: 128 for APAR_BF16 and APAR_BF16_FP8KV; 64 or 128 for APAR_F32 */
    int32_t block_size;  /* tokens per KV block; must be 16                              */
    int32_t dtype;       /* APAR_F32, APAR_BF16 or APAR_BF16_FP8KV (bf16 at the interface) */
    int32_t max_threads; /* upper bound on ids ever issued by this pool                  */
    int64_t num_blocks;  /* N: blocks in the pool, at most 2^26                          */
    float softmax_scale; /* 0 means 1/sqrt(head_dim)                                     */
} apar_pool_config;

typedef struct apar_stats {
    int64_t total_blocks;
    int64_t used_blocks;    /* blocks with refcount > 0                                  */
    int64_t free_blocks;
    int64_t live_threads;
    int64_t threads_issued;
    int64_t cow_copies;     /* copy-on-write block copies since creation                 */
    int64_t block_bytes;    /* 2 * Hkv * 16 * d * element size                           */
    int64_t bytes_resident; /* used_blocks * block_bytes                                 */
    int64_t bytes_vanilla;  /* sum over live threads of ceil(len/16) * block_bytes: what */
                            /* a layout that copies the prefix on every fork would hold  */
                            /* (the paper's contiguous-cache setting, App. C.1)          */
} apar_stats;

/* What the last apar_decode_attention[_spec] call on this pool scheduled. */
typedef struct apar_plan_info {
    int64_t n_threads;         /* listed threads                                         */
    int64_t n_segments;        /* maximal runs of blocks shared by one set of threads    */
    int64_t n_units;           /* workgroups launched (plan workgroups x kv heads)        */
    int64_t n_partial_rows;    /* (unit, thread) partial results merged afterwards       */
    int64_t unique_blocks;     /* distinct blocks read                                   */
    int64_t unique_tokens;     /* filled slots in those blocks: each cached row once     */
    int64_t path_tokens;       /* sum of the listed threads' lengths                     */
    int64_t algorithmic_bytes; /* unique_tokens * 2*Hkv*d*e + q read + output written    */
                               /* (+ candidates' k, v for the multi-candidate call); on  */
                               /* an fp8 pool the tokens of full blocks count 1 byte per */
                               /* element plus 8 bytes of scales per (block, kv head)    */
} apar_plan_info;

/* Device time measured with HIP events on the caller's stream while profiling is on. */
typedef struct apar_profile {
    int64_t n_decode_calls;
    double attention_kernel_ms; /* sum over calls: the partial-attention kernel           */
    double merge_kernel_ms;     /* sum over calls: the merge / normalise kernel            */
    double plan_host_ms;        /* sum over calls: host time building + staging the plan,
                                   without the waits counted in host_wait_ms               */
    int64_t n_append_calls;
    double append_kernels_ms;   /* sum over calls: copy-on-write copies + row writes       */
    double host_wait_ms;        /* sum over decode and append calls: host time spent waiting
                                   for a staging buffer that the GPU had not consumed yet,
                                   i.e. the GPU was the slower side                        */
} apar_profile;

/*
 * Create a pool over caller-owned device memory.
 *   kv_dev/kv_bytes : device buffer of at least num_blocks * block_bytes bytes,
 *                     256-byte aligned; contents need not be initialised.
 * kv_dev == NULL with kv_bytes == 0 creates a DRY-RUN pool: it keeps the same
 * books (tables, refcounts, free list) and builds the same plans, but owns no
 * device memory and launches nothing, e.g. to size a pool from a trace.  On a
 * dry-run pool every *_dev argument of the other calls must be NULL and
 * apar_read_kv_rows is an error; no call of it touches the GPU.
 * Errors: INVALID_ARG (null pointers, block_size != 16, heads not divisible,
 * num_blocks out of range, buffer too small or misaligned), UNSUPPORTED
 * (head_dim / dtype combination), HIP.
 */
APAR_API int apar_pool_create(const apar_pool_config* cfg, void* kv_dev, size_t kv_bytes, apar_pool** out);

/* Waits for the pool's outstanding device work, frees bookkeeping and staging
 * memory (never the KV buffer).  NULL is accepted. */
APAR_API int apar_pool_destroy(apar_pool* pool);

/* A new empty root thread (the prompt sequence that starts a sequence group,
 * Alg. 1).  Errors: THREAD_CAPACITY. */
APAR_API int apar_thread_create(apar_pool* pool, apar_thread* out);

/*
 * Fork (Alg. 1: a sequence that ends in [Fork] spawns a copy of itself; Sec. 2.3): n_children new threads whose table and
 * length equal the parent's; every block the parent holds gains n_children
 * references.  Allocates no block and copies nothing; the copy of a shared,
 * partly filled tail block is deferred to the first append that needs it.  The
 * parent stays live until freed.  children_out receives n_children
 * consecutive ids.  Errors: INVALID_THREAD, INVALID_ARG (n_children < 1),
 * THREAD_CAPACITY.
 */
APAR_API int apar_fork(apar_pool* pool, apar_thread parent, int n_children, apar_thread* children_out);

/*
 * Append n_tokens rows to one thread (Alg. 1: s.append_token).
 *   k_dev, v_dev : [n_tokens, Hkv, d], pool dtype, row-major, contiguous.
 * Token by token: at a block boundary a fresh block is taken; otherwise a tail
 * block that other threads also hold is first copied to a fresh block
 * (copy-on-write; at most one copy per call), then the row is written.
 * n_tokens == 0 is a no-op.  Errors: INVALID_THREAD, INVALID_ARG,
 * OUT_OF_BLOCKS (checked before anything changes), HIP.
 */
APAR_API int apar_append_kv(apar_pool* pool, apar_thread thread, const void* k_dev, const void* v_dev,
                   int n_tokens, void* hip_stream);

/* One row for each listed thread, processed in list order (a thread may be
 * listed more than once).  k_dev, v_dev: [n, Hkv, d]. */
APAR_API int apar_append_kv_batch(apar_pool* pool, const apar_thread* threads, int n, const void* k_dev,
                         const void* v_dev, void* hip_stream);

/*
 * Decode attention (Sec. 2.2 "Training attention", Sec. 2.4 feature 3).  For
 * listed thread i and query head h:
 *   out[i,h] = sum_j softmax_j(scale * <q[i,h], K_j[h / (Hq/Hkv)]>) * V_j[h / (Hq/Hkv)]
 * with j over all len(threads[i]) rows reachable through that thread's table
 * (its ancestors' rows up to each fork point and its own rows, the newest
 * included).  Blocks shared by several listed threads are read once and
 * applied to all of their queries.
 *   q_dev, out_dev : [n, Hq, d], pool dtype.   threads : host array of n ids
 *   (duplicates allowed).  n == 0 is a no-op.
 * Errors: INVALID_THREAD, INVALID_ARG (null pointers, n < 0, or a listed
 * thread of length 0: softmax over no rows is undefined), HIP.
 */
APAR_API int apar_decode_attention(apar_pool* pool, const void* q_dev, const apar_thread* threads, int n,
                          void* out_dev, void* hip_stream);

/*
 * Multi-candidate decode attention (verification step of speculative decoding
 * with tree attention, Sec. 3.2 Medusa-APAR, App. C.1).  Every listed thread
 * carries n_cand candidate tokens; candidate c attends to all cached rows of
 * the thread and to candidate c' iff bit c' of mask_dev[i*n_cand + c] is set
 * (every row must have its own bit set).  Candidates' K, V are not cached by
 * this call; append the accepted ones afterwards.
 *   q_dev, out_dev : [n, n_cand, Hq, d];  cand_k_dev, cand_v_dev : [n, n_cand, Hkv, d];
 *   mask_dev : [n, n_cand] uint8;  1 <= n_cand <= 8.
 */
APAR_API int apar_decode_attention_spec(apar_pool* pool, const void* q_dev, const void* cand_k_dev,
                               const void* cand_v_dev, const uint8_t* mask_dev, int n_cand,
                               const apar_thread* threads, int n, void* out_dev, void* hip_stream);
/*
 * apar_decode_attention for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result, same kernels - but
 * the call's plan tables and partial results live in a workspace of fixed size that is part of the
 * library's device image (one copy per GPU, held until the process ends) instead of in memory the
 * library allocates, every kernel runs on `hip_stream` itself, and the call creates no stream or
 * event and is never profiled.  It calls no hipMalloc, hipFree, hipHostMalloc or any other
 * allocating routine (what it needs besides - the workspace's address on the pool's device, a
 * pinned staging buffer of APAR_FIXED_PLAN_BYTES and one event - apar_pool_create obtained).
 * Limits: the staged plan (128 bytes per workgroup, 8 per block read, 8 per listed thread and 4
 * per partial result to merge) must fit APAR_FIXED_PLAN_BYTES, and the partial results
 * ((head_dim + 2) floats per (partial row, q head); none when every sharing subtree fits one work
 * unit) APAR_FIXED_PARTIAL_BYTES; beyond either the call returns APAR_ERR_WORKSPACE_LIMIT and
 * enqueues nothing.  The host may wait for the previous fixed call's plan upload (not for its kernels).
 * All pools on one GPU share that GPU's workspace, which keeps the last call's contents: nothing
 * in it has to start at zero (a call overwrites every table and every partial result it reads),
 * but two fixed calls that overlap on one GPU - different streams, or different pools, without an
 * order between them - race on it.  Calls on one stream are ordered by the stream.
 * Errors: as apar_decode_attention, plus WORKSPACE_LIMIT, and INVALID_ARG on a dry-run pool.
 */
#define APAR_FIXED_PLAN_BYTES (2 << 20)
#define APAR_FIXED_PARTIAL_BYTES (6 << 20)
APAR_API int apar_decode_attention_fixed(apar_pool* pool, const void* q_dev, const apar_thread* threads, int n,
                                void* out_dev, void* hip_stream);

/* As apar_append_kv_batch, but row i of the call is read from row src_rows[i] (>= 0, host array) of
 * k_dev, v_dev, so that a caller can append a subset of a larger array of rows without gathering it
 * first (Alg. 1 batches the rows of many sequence groups; a scheduler may have dropped some). */
APAR_API int apar_append_kv_gather(apar_pool* pool, const apar_thread* threads, const int32_t* src_rows, int n,
                          const void* k_dev, const void* v_dev, void* hip_stream);

/*
 * Commit of a multi-candidate step: the accepted candidates become part of each thread's
 * sequence (Sec. 3.2, the Medusa-APAR setting: a predict-verify step keeps one root path of
 * its candidate tree; App. C.1: sequences accept different numbers of tokens and mis-predicted
 * slots do not count).
 * For every listed thread i, in listed order, the candidates c whose bit is set in
 * accept_masks[i] are appended in ascending c (a candidate's ancestors have smaller indices,
 * so this is root -> accepted node order), their rows taken straight from
 *   cand_k_dev, cand_v_dev : [n, n_cand, Hkv, d], device, pool dtype
 * - the arrays the preceding apar_decode_attention_spec call was given - with no gather on
 * the caller's side and no second pass.  Tables, refcounts and the free list end up exactly as
 * after apar_append_kv_batch with thread i repeated once per accepted candidate.
 *   accept_masks : [n] bytes, HOST memory (the host books need them); bits >= n_cand must be 0.
 * A thread may be listed more than once and a mask may be 0.  All or nothing.
 * Errors: INVALID_ARG (null pointers, n_cand outside 1..8, a bit for a missing candidate),
 * INVALID_THREAD, OUT_OF_BLOCKS, HIP.
 */
APAR_API int apar_commit_candidates(apar_pool* pool, const apar_thread* threads, int n, const void* cand_k_dev,
                           const void* cand_v_dev, int n_cand, const uint8_t* accept_masks, void* hip_stream);

/*
 * Prefill attention under the paragraph-tree mask (Sec. 2.2 "Training attention", Fig. 2: a token
 * attends only to the tokens on its path to the root, causally; the same mask serves the prefill of
 * a prompt or of a whole segment at inference).  The last m[i] cached rows of listed thread i are
 * its query tokens' own rows - append them first -: query r (0 <= r < m[i]) sits at position
 * len_i - m[i] + r and attends to rows 0 .. that position of the thread, i.e. to its ancestors'
 * rows up to each fork point and to its own rows up to and including itself.  Listing every node
 * of a paragraph tree, each with its own segment length as m, computes the attention of the whole
 * tree in one call; m[i] = 1 is the decode step.
 *   q_dev, out_dev : [sum(m), Hq, d], pool dtype, device; thread 0's m[0] query tokens first.
 *   threads, m     : host arrays of n entries (a thread may be listed more than once).
 * Only pools whose Hq / Hkv divides 16 are supported.  Nothing is written but out_dev.
 * Errors: INVALID_THREAD, INVALID_ARG (null pointers, m[i] outside 1..len_i), UNSUPPORTED, HIP.
 */
APAR_API int apar_prefill_attention(apar_pool* pool, const void* q_dev, const apar_thread* threads, const int32_t* m,
                           int n, void* out_dev, void* hip_stream);

/* Release (Alg. 1 ReleaseCache): walks the table from its last block to its
 * first, drops one reference from each and returns a block to the pool when no
 * thread holds it any more.  Errors: INVALID_THREAD. */
APAR_API int apar_free_thread(apar_pool* pool, apar_thread thread);

/* ---- introspection (parity checks and reports) -------------------------- */
APAR_API int apar_thread_len(apar_pool* pool, apar_thread thread, int64_t* len_out);
/* Copies up to cap ids into table_out and stores the table length in n_out
 * (INVALID_ARG if cap is too small; n_out is still set). */
APAR_API int apar_thread_block_table(apar_pool* pool, apar_thread thread, int32_t* table_out, int cap, int* n_out);
APAR_API int apar_block_refcount(apar_pool* pool, int32_t block, int32_t* refcount_out);
APAR_API int apar_pool_stats(apar_pool* pool, apar_stats* out);
APAR_API int apar_last_plan_info(apar_pool* pool, apar_plan_info* out);
/* Gathers rows [first, first+n) of a thread out of the pool's private layout
 * into row-major k_out_dev, v_out_dev : [n, Hkv, d]. */
APAR_API int apar_read_kv_rows(apar_pool* pool, apar_thread thread, int64_t first, int n, void* k_out_dev,
                      void* v_out_dev, void* hip_stream);

/* ---- decoding controller (Alg. 1) ---------------------------------------
 * One sequence group per prompt (Sec. 2.3).  The controller keeps each sequence's
 * tokens, the paragraph tree (Sec. 2.2: a node points at a slice of a sequence and
 * has a first-child and a next-sibling pointer) and applies one decoding step of
 * Alg. 1 to the tokens the caller sampled.  It samples nothing and runs no model:
 * per step the caller lists the unfinished sequences (apar_group_unfinished), runs
 * apar_decode_attention over them, draws one token per sequence and calls
 * apar_group_step.  Token ids >= 0 are ordinary tokens. */
typedef struct apar_group apar_group;
enum { APAR_TOKEN_FORK = -1, APAR_TOKEN_CHILD = -2, APAR_TOKEN_EOS = -3 };

typedef struct apar_group_step_info {
    int32_t n_forked;        /* sequences whose last token was [Fork]: each spawned one child      */
    int32_t n_finished;      /* sequences that sampled [EOS] and were released                     */
    int32_t n_rows_appended; /* K,V rows consumed from k_dev / v_dev                               */
    int32_t n_unfinished;    /* unfinished sequences after the step (children included)            */
} apar_group_step_info;

typedef struct apar_group_info {
    int64_t n_sequences, n_unfinished, n_nodes, steps;
    int64_t prompt_tokens;
    int64_t generated_tokens;  /* sampled tokens (injected [Child] tokens not counted)              */
    int64_t attended_tokens;   /* sum over sampled tokens of the tokens attended to when predicting */
                               /* them (Sec. 3.4 "Attended tokens")                                 */
    int64_t cached_tokens;     /* KV slots needed now, in tokens: shared prefixes once, released    */
                               /* sequences only as far as a live thread still shares them          */
    int64_t max_cached_tokens; /* maximum of cached_tokens over the steps so far (Sec. 3.4)         */
} apar_group_info;

/* Starts a group: a root sequence holding the prompt (n_prompt >= 1 rows in k_dev, v_dev:
 * [n_prompt, Hkv, d]) and the root paragraph node, which starts where the prompt ends.  Errors as
 * apar_thread_create and apar_append_kv; nothing is left behind on failure. */
APAR_API int apar_group_create(apar_pool* pool, const int32_t* prompt_tokens, int n_prompt, const void* k_dev,
                               const void* v_dev, void* hip_stream, apar_group** out);
/* Releases the sequences that are still unfinished and frees the group.  NULL is accepted. */
APAR_API int apar_group_destroy(apar_group* group);
/* Thread ids of the unfinished sequences, in creation order; n_out is always set. */
APAR_API int apar_group_unfinished(apar_group* group, apar_thread* threads_out, int cap, int* n_out);
/*
 * One decoding step of Alg. 1.  sampled[i] is the token drawn for the i-th unfinished sequence s
 * (the order of apar_group_unfinished; n must equal their number).  For each s in order: if
 * s ends in [Fork], s is forked, [Child] is appended to the new sequence, s's open paragraph node is
 * closed and two nodes are opened: the new sequence's as its first child, s's next one as its next sibling; then sampled[i]
 * is appended to s; if it is [EOS], s is finished and its cache released.  A child joins the
 * group's list from the next step on.  k_dev, v_dev: one row per appended token, in this order:
 * for each s in order, the [Child] row of its new thread if it forks, then the row of sampled[i].
 * Errors: INVALID_ARG (wrong n, a sampled [Child]), THREAD_CAPACITY, OUT_OF_BLOCKS, HIP; on error
 * the group and the pool are unchanged.
 */
APAR_API int apar_group_step(apar_group* group, const int32_t* sampled, int n, const void* k_dev,
                             const void* v_dev, void* hip_stream, apar_group_step_info* info_out);
/* Restore(r) of Alg. 1: the generated tokens in root / first-child / next-sibling order
 * (the prompt and the injected [Child] tokens are not part of any node).  n_out is always set;
 * INVALID_ARG if cap is too small. */
APAR_API int apar_group_restore(apar_group* group, int32_t* tokens_out, int64_t cap, int64_t* n_out);
APAR_API int apar_group_get_info(apar_group* group, apar_group_info* out);

/* ---- serving loop (Sec. 3.3 "Results in High-Throughput Scenarios", App. C.2) -------------
 * Requests wait in a first-come-first-served queue over one pool.  Per decode step the caller
 * admits (apar_server_admit), lists the batch (apar_server_batch), runs apar_decode_attention
 * over its threads, samples one token per entry and applies one decoding step of Alg. 1 to every running
 * request at once (apar_server_step): forks, one batched append of all rows, early release of
 * every sequence that drew [EOS] (Sec. 2.4 feature 2) and collection of completed requests.  The
 * paper serves through an existing paged-attention engine and says only that concurrency is
 * capped and that over-admission leads to swapping or recomputation of KV cache; the policy here:
 *   admission  - head of the queue only, while fewer than max_running requests run and
 *                free_blocks - ceil(prompt / 16) >= watermark_blocks;
 *   preemption - when a step's rows do not fit, the most recently admitted running request is
 *                released and goes back to the head of the queue (it restarts from its prompt:
 *                recomputation), and the step is retried without it until it fits.  The oldest running
 *                request is never released: when the step does not fit with it alone, the pool is too
 *                small for that request and apar_server_step returns OUT_OF_BLOCKS. */
typedef struct apar_server apar_server;
typedef struct apar_server_config {
    int32_t max_running;
    int32_t watermark_blocks;
} apar_server_config;
typedef struct apar_server_seq {   /* one unfinished sequence of the batch */
    int32_t request_id;
    apar_thread thread;
    int32_t seq_index;    /* index of the sequence in its group, creation order (0: the prompt's)  */
    int32_t last_token;
    int64_t length;       /* tokens so far, prompt included                                          */
    int64_t start_len;    /* length it began with: the prompt (root) or parent's tokens + [Child]    */
    int32_t group_size;   /* sequences its group has issued so far                                   */
    int32_t reserved;
} apar_server_seq;
typedef struct apar_server_step_info {
    int32_t n_preempted, n_forked, n_finished_sequences, n_finished_requests, n_rows_appended, n_running;
} apar_server_step_info;
typedef struct apar_server_stats {
    int64_t steps, n_submitted, n_waiting, n_running, n_finished, n_admissions, n_preemptions;
    int64_t generated_tokens;        /* sampled tokens of steps that were applied (a preempted request's count again) */
    int64_t batch_sequences_total;   /* sum over steps of the sequences decoded                      */
    int64_t peak_used_blocks, peak_running, peak_threads;
} apar_server_stats;
APAR_API int apar_server_create(apar_pool* pool, const apar_server_config* cfg, apar_server** out);
/* Releases whatever still runs.  NULL is accepted. */
APAR_API int apar_server_destroy(apar_server* server);
APAR_API int apar_server_submit(apar_server* server, int32_t request_id, const int32_t* prompt_tokens, int n_prompt);
/* Admits from the head of the queue.  The j-th request admitted by the call takes its prompt's rows
 * from k_dev, v_dev ([rows_available, Hkv, d]) right after those of the (j-1)-th; admission also stops
 * before a prompt that no longer fits in rows_available.  Both NULL on a dry-run pool. */
APAR_API int apar_server_admit(apar_server* server, const void* k_dev, const void* v_dev, int64_t rows_available,
                               void* hip_stream, int32_t* n_admitted_out, int64_t* rows_used_out);
/* The unfinished sequences of all running requests: requests in admission order, sequences in
 * creation order.  n_out is always set; INVALID_ARG if cap is too small. */
APAR_API int apar_server_batch(apar_server* server, apar_server_seq* out, int cap, int* n_out);
/* sampled[i]: the token drawn for batch entry i (n = batch size).  k_dev, v_dev: the rows of the
 * step, request by request in batch order, each request's rows as in apar_group_step.  The entries
 * and rows of a request preempted by this call are skipped.  Errors: INVALID_ARG, THREAD_CAPACITY,
 * HIP, and OUT_OF_BLOCKS when the step does not fit even with the oldest running request alone; then
 * no step was applied (requests preempted before the error stay preempted). */
APAR_API int apar_server_step(apar_server* server, const int32_t* sampled, int n, const void* k_dev, const void* v_dev,
                              void* hip_stream, apar_server_step_info* info_out);
/* The oldest completed request: its id (-1 if none), its tokens in Restore order (Alg. 1) and its
 * Sec. 3.4 counters.  INVALID_ARG with n_tokens_out set if cap is too small (the request stays). */
APAR_API int apar_server_pop_finished(apar_server* server, int32_t* request_id_out, int32_t* tokens_out, int64_t cap,
                                      int64_t* n_tokens_out, apar_group_info* info_out);
APAR_API int apar_server_get_stats(apar_server* server, apar_server_stats* out);

/* ---- measurement -------------------------------------------------------- */
/* While on, every decode and append call brackets its kernels with HIP events. */
APAR_API int apar_profile_enable(apar_pool* pool, int on);
/* Waits for the recorded events, adds up the elapsed times since the last
 * read, stores them in out and resets the sums. */
APAR_API int apar_profile_read(apar_pool* pool, apar_profile* out);
/* Per-call device times (ms) of the attention kernel for the decode calls that the most recent
 * apar_profile_read summed, in call order, so that a caller can report a median and percentiles.
 * Stores the count in n_out; INVALID_ARG if cap is too small (n_out is still set). */
APAR_API int apar_profile_attention_calls(apar_pool* pool, float* ms_out, int64_t cap, int64_t* n_out);

/* ---- testing and tuning ---------------------------------------------------
 * Everything in this section exists for the test-suite and for experiments.  It is NOT part of the
 * stable interface: the knobs steer internal policies whose defaults are the product, and the plan
 * export hands out the kernels' private tables, whose layout changes with the kernels.
 * APAR_PLAN_RECORD_VERSION names the layout documented below; apar_plan_record_version() returns the
 * one the loaded library was built with, so that a reader of the tables can refuse a layout it does
 * not know. */
#define APAR_PLAN_RECORD_VERSION 2
APAR_API int apar_plan_record_version(void);
/* Tables of the last decode call's plan, for inspection (int32 arrays).  The listed threads are
 * numbered depth-first along their sharing tree ("rank"); a thread's query rows are cut into
 * `slices` slices of at most 16 rows, and row group = rank * slices + slice.  `which`:
 *   APAR_PLAN_WORKGROUPS  32 ints per workgroup: [0] first shared tile, [1] shared tile count,
 *                         [2] row group the shared tiles' ranges are relative to, [3] bits 0-7: 16-row tiles per wavefront
 *                         (1 or 2), or 32 for a matrix unit - a stand-alone chunk of a shared segment for up to 128
 *                         rows of whole threads, all named by wavefront entry 0, the other entries empty -
 *                         (workgroups are stored 32 first, then 2, then 1), bits 8-31: how many
 *                         of the shared tiles are full (every list holds its full tiles first), then
 *                         4 wavefronts x 6: first own tile, own tile count, first row group, row
 *                         group count, first partial-result row (of the thread owning the first
 *                         row group), flags (bit 0: writes output rows directly); [28..31] full tiles at the head
 *                         of each wavefront's own list;
 *   APAR_PLAN_TILES       2 ints per tile: block id, lo | hi << 10 | filled_slots << 20, where
 *                         [lo, hi) are the row groups the block applies to, relative to the
 *                         wavefront's first row group (own tiles) or to [2] (shared tiles);
 *   APAR_PLAN_DFS_THREADS rank -> index into the listed threads;
 *   APAR_PLAN_PATH_OFS    [n+1] offsets into PATH_IDS by listed index;  APAR_PLAN_PATH_IDS  the
 *                         partial-result rows merged for each listed thread (none: written directly);
 *   APAR_PLAN_GEOMETRY    rows per thread, rows per slice, slices;
 *   APAR_PLAN_CHANGED_WORKGROUP_WORDS, APAR_PLAN_CHANGED_TILE_WORDS  if the last call carried its plan over
 *                         (apar_set_plan_reuse): which ints of the two tables it changed - the ints it rewrites
 *                         in the copy of the tables on the device, every other int staying as the previous call
 *                         left it (an int may be named twice); empty after a call that built its plan.
 * Stores the element count in n_out; INVALID_ARG if cap is too small. */
enum { APAR_PLAN_WORKGROUPS = 0, APAR_PLAN_TILES = 1, APAR_PLAN_DFS_THREADS = 2, APAR_PLAN_PATH_OFS = 3,
       APAR_PLAN_PATH_IDS = 4, APAR_PLAN_GEOMETRY = 5, APAR_PLAN_CHANGED_WORKGROUP_WORDS = 6,
       APAR_PLAN_CHANGED_TILE_WORDS = 7 };
APAR_API int apar_last_plan_export(apar_pool* pool, int which, int32_t* out, int64_t cap, int64_t* n_out);
/* Tuning knob: the most blocks one wavefront is given in one work unit (1..65536; default 512).
 * Sharing subtrees with more blocks than that are cut into several units whose partial results are
 * merged afterwards; small values exist to exercise that path. */
APAR_API int apar_set_chunk_blocks(apar_pool* pool, int blocks_per_unit);
/* Tuning knob (bf16 pools): a shared segment that stands alone as a unit - its holders have more query rows
 * than one fused workgroup carries (128) - goes to the 32x32 matrix-core kernel, up to 128 rows per workgroup,
 * when its holders bring at least min_rows query rows (candidates x q heads per kv head x threads; default 256)
 * and it has at least min_blocks blocks (default 128; shorter ones are cheaper read again by every unit below,
 * see apar_set_inline_shared).
 * Matrix units are launched ahead of the other units of a call, not beside them.  min_rows = 0 keeps every unit on the row-tile kernel; (1, 1) sends every such segment
 * to the matrix kernel.  Results agree to rounding.  fp32 pools ignore the knob. */
APAR_API int apar_set_matrix_units(apar_pool* pool, int min_rows, int min_blocks);
/* Tuning knob: what happens to a sharing subtree whose threads bring more query rows than one unit carries
 * (128) and whose top segment does not go to the matrix kernel.  On (default): its threads, in depth-first
 * order, are cut into full units of consecutive threads, and every unit reads the segments above its
 * threads again - no partial results, no merge; used when nothing above leaves partial results and no unit
 * would read more blocks than four times the unit cap.  Off: the top segment stands alone with one partial
 * result per (chunk, thread) and its children are tried again. */
APAR_API int apar_set_inline_shared(apar_pool* pool, int on);
/* Tuning knob: which kernel apar_prefill_attention runs on a bf16 pool.  ROW_TILES is the decode kernel
 * under a prefill plan (16-row tiles; a prefix shared by sibling threads is read once for all of them),
 * MATRIX the 32x32 matrix-core kernel (one workgroup per thread and chunk of 128 query rows; needs a
 * group size that divides 16, otherwise the call stays on ROW_TILES).  AUTO (default) takes MATRIX when
 * a query token attends to 1024 rows or more on average.  Both give the same result to rounding.
 * fp32 pools ignore the knob.  apar_last_prefill_kernel tells which one the most recent call ran (0: none). */
enum { APAR_PREFILL_AUTO = 0, APAR_PREFILL_ROW_TILES = 1, APAR_PREFILL_MATRIX = 2 };
APAR_API int apar_set_prefill_kernel(apar_pool* pool, int which);
APAR_API int apar_last_prefill_kernel(apar_pool* pool);

/* Write checks (off by default).  While on, every call that is about to launch kernels writing KV
 * blocks - appended rows, copy-on-write copies, the re-layout of a block that just became full -
 * first verifies on the host that each destination block is held by exactly one thread (Sec. 2.3: a
 * block that several sequences share is never written; the writer copies it first).  A violation is
 * a bug in the library's bookkeeping: the call returns APAR_ERR_INTERNAL and launches nothing.  The
 * check runs on bookkeeping-only pools as well. */
APAR_API int apar_set_write_checks(apar_pool* pool, int on);

/* Plans carried over (on by default).  A decode call that lists, position by position, the threads of the
 * previous decode call on the pool - or threads forked from them since - with the same candidate count does
 * not build its plan afresh: the previous one is brought up to date along each thread's last blocks (fill
 * counts, a copy-on-write copy in place of the block it copied, one new block per thread) - the per-step
 * loop of Alg. 1 changes nothing else between two steps.  Any other change (another set of threads, a
 * thread appended to while it shares its last blocks with another listed thread, more than one new block
 * for a thread, a knob of this section moved) makes the call build a new plan, as does turning this off.
 * Both kinds of plan read exactly the listed threads' tables; apar_plan_info describes the plan that ran,
 * its n_segments as counted when it was last built.  apar_plan_counts: decode calls so far that built
 * their plan, and that carried one over. */
APAR_API int apar_set_plan_reuse(apar_pool* pool, int on);
APAR_API int apar_plan_counts(apar_pool* pool, int64_t* n_built, int64_t* n_carried);

APAR_API const char* apar_status_string(int status);
/* Text of the last HIP error seen on this host thread by the library ("" if none). */
APAR_API const char* apar_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* APAR_H */
