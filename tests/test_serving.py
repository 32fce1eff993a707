"""The serving loop (queue, admission, early release, preemption) of the library against the plain-Python
oracle loop, on bookkeeping-only pools (CPU)."""
import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import SamplerConfig, make_requests, sample_flat, sample_tokens
from oracle import BlockLedger
from oracle.serving import ServingOracle
from paper_2401_06761_amd.serving import ServingRun

from harness import books_equal

CFG = SamplerConfig(p_fork=0.05, p_eos=0.02, max_threads=6, min_new=12, max_len=260)


def _oracle_run(reqs, n_blocks, max_running, watermark, flat=None, check=None):
    led = BlockLedger(n_blocks, max_threads=1 << 30)
    o = ServingOracle(led, max_running, watermark)
    by = {r.rid: r for r in reqs}
    for r in reqs:
        o.submit(r.rid, r.prompt_tokens())
    trace = []
    while True:
        adm = o.admit()
        b = o.batch()
        if not b:
            assert not o.waiting
            break
        seeds = [by[e["request_id"]].seed for e in b]
        if flat is None:
            xs = sample_tokens(CFG, seeds, [e["seq_index"] for e in b], [e["length"] for e in b],
                               [e["last_token"] for e in b], [e["start_len"] for e in b], [e["group_size"] for e in b])
        else:
            xs = sample_flat(CFG, seeds, [e["length"] for e in b], [flat[e["request_id"]] for e in b])
        info = o.step(xs.tolist())
        trace.append({"admitted": len(adm), "threads": [e["thread"] for e in b], "sampled": xs.tolist(),
                      "n_preempted": info["n_preempted"], "n_forked": info["n_forked"],
                      "n_rows_appended": info["n_rows_appended"], "n_finished_requests": info["n_finished_requests"]})
        if check is not None:
            check(len(trace), led)
    return o, led, trace


def _decode_alone(req):
    """One request through Algorithm 1 with nothing else around: what its response must be under any schedule,
    because the sampler depends on (request seed, sequence index, sequence length) only."""
    from oracle.controller import SequenceGroup

    g = SequenceGroup(req.prompt_tokens())
    start = {0: req.prompt_len}
    steps = 0
    while not g.is_finished():
        todo = g.unfinished()
        xs = sample_tokens(CFG, [req.seed] * len(todo), [s.sid for s in todo], [len(s.tokens) for s in todo],
                           [s.last_token for s in todo], [start[s.sid] for s in todo], [len(g.G)] * len(todo))
        before = len(g.G)
        g.step(xs.tolist())
        for c in g.G[before:]:
            start[c.sid] = len(c.tokens)
        steps += 1
    return g.restore(), steps, g


@pytest.mark.parametrize("n_blocks,max_running,watermark", [(4096, 64, 0), (4096, 5, 0), (160, 12, 2), (96, 40, 0), (64, 8, 4)])
def test_oracle_loop_against_what_the_policy_fixes(n_blocks, max_running, watermark):
    """The oracle's loop alone, against facts that do not come from it: every response equals the request
    decoded alone (whatever was preempted and restarted); requests are admitted in submission order and
    never overtake; the pool, the watermark and the cap on running requests are respected at every step;
    with room for everything nothing is preempted and the loop takes as many steps as the longest request;
    the books are empty at the end."""
    reqs = make_requests(24, seed=n_blocks + max_running, prompt_lo=8, prompt_hi=120)
    by = {r.rid: r for r in reqs}
    alone = {r.rid: _decode_alone(r) for r in reqs}
    order_of = {r.rid: i for i, r in enumerate(reqs)}
    seen = {"max_used": 0}

    def check(step, led):
        led.check_invariants()
        assert led.used_blocks() <= n_blocks
        seen["max_used"] = max(seen["max_used"], led.used_blocks())

    led = BlockLedger(n_blocks, max_threads=1 << 30)
    o = ServingOracle(led, max_running, watermark)
    for r in reqs:
        o.submit(r.rid, r.prompt_tokens())
    done_before = set()
    while True:
        free_before = led.free_blocks()
        adm = o.admit()
        # admission: queue order, and each one left the watermark standing
        free = free_before
        for rid in adm:
            free -= (by[rid].prompt_len + 15) // 16
            assert free >= watermark
        assert free == led.free_blocks()
        running = [r["rid"] for r in o.running]
        assert len(running) <= max_running
        # no overtaking: whoever runs or is done was submitted before everybody still waiting
        waiting = [rid for _, rid, _ in o.waiting]
        if waiting:
            first_waiting = min(order_of[rid] for rid in waiting)
            assert all(order_of[rid] < first_waiting for rid in running)
            assert [order_of[rid] for rid in waiting] == sorted(order_of[rid] for rid in waiting)
        b = o.batch()
        if not b:
            assert not o.waiting
            break
        seeds = [by[e["request_id"]].seed for e in b]
        xs = sample_tokens(CFG, seeds, [e["seq_index"] for e in b], [e["length"] for e in b],
                           [e["last_token"] for e in b], [e["start_len"] for e in b], [e["group_size"] for e in b])
        o.step(xs.tolist())
        check(o.steps, led)
    assert sorted(rid for rid, _, _ in o.finished) == sorted(by)
    for rid, toks, g in o.finished:
        want, _, g_alone = alone[rid]
        assert toks == want, f"request {rid}"
        assert (g.attended, g.generated, g.max_cached) == (g_alone.attended, g_alone.generated, g_alone.max_cached)
    assert led.used_blocks() == 0
    if n_blocks == 4096:
        assert o.preemptions == 0 and o.admissions == len(reqs)
        if max_running >= len(reqs):
            assert o.steps == max(steps for _, steps, _ in alone.values())
            assert o.generated == sum(g.generated for _, _, g in alone.values())
    else:
        assert o.preemptions > 0 and o.admissions == len(reqs) + o.preemptions
        assert o.generated > sum(g.generated for _, _, g in alone.values())  # restarted work is counted


@pytest.mark.parametrize("n_blocks,max_running,watermark", [(4096, 64, 0), (160, 12, 2), (96, 40, 0), (64, 8, 4)])
def test_serving_loop_matches_oracle_step_by_step(n_blocks, max_running, watermark):
    reqs = make_requests(24, seed=n_blocks, prompt_lo=8, prompt_hi=120)
    pool = ap.Pool(4, 2, 64, "f32", n_blocks, max_threads=1 << 30, dry_run=True)
    run = ServingRun(pool, reqs, CFG, max_running, watermark)
    run.keep_trace = True
    stats = run.run()
    o, led, trace = _oracle_run(reqs, n_blocks, max_running, watermark)
    assert run.trace == trace
    assert run.outputs == {rid: toks for rid, toks, _ in o.finished}
    assert sorted(run.outputs) == [r.rid for r in reqs]           # everybody completes
    assert [rid for rid, _, _ in o.finished] == list(run.outputs)  # in the same order
    for rid, _, g in o.finished:
        gi = run.infos[rid]
        assert (gi.max_cached_tokens, gi.attended_tokens, gi.generated_tokens) == (g.max_cached, g.attended, g.generated)
    assert (stats["steps"], stats["preemptions"], stats["admissions"]) == (o.steps, o.preemptions, o.admissions)
    assert stats["peak_used_blocks"] == o.peak_used and stats["peak_threads"] == o.peak_threads
    assert stats["generated_tokens"] == o.generated
    if n_blocks <= 160:
        assert stats["preemptions"] > 0   # these pools are tight on purpose
    books_equal(pool.handle, led)
    assert ap.apar_pool_stats(pool.handle).used_blocks == 0
    run.close()
    pool.close()


def test_books_agree_after_every_step_under_preemption():
    reqs = make_requests(10, seed=3, prompt_lo=8, prompt_hi=100)
    pool = ap.Pool(4, 2, 64, "f32", 48, max_threads=1 << 30, dry_run=True)
    run = ServingRun(pool, reqs, CFG, 6, 1)
    snapshots = []

    def check(step, led):
        # advance the library to the same step and compare the books
        while len(snapshots) < step:
            assert run.step()
            snapshots.append(1)
        books_equal(pool.handle, led)

    o, led, trace = _oracle_run(reqs, 48, 6, 1, check=check)
    assert o.preemptions > 0
    run.close()
    pool.close()


def test_flat_stand_in_needs_more_steps_and_more_cache_for_the_same_responses():
    # the same responses decoded sequentially: one sequence per request, as long as prompt + output
    reqs = make_requests(16, seed=9, prompt_lo=8, prompt_hi=64)
    big = 4096
    pool = ap.Pool(4, 2, 64, "f32", big, max_threads=1 << 30, dry_run=True)
    a = ServingRun(pool, reqs, CFG, 16, 0)
    sa = a.run()
    a.close()
    flat = {r.rid: r.prompt_len + len(a.outputs[r.rid]) for r in reqs}
    b = ServingRun(pool, reqs, CFG, 16, 0, flat_lengths=flat)
    sb = b.run()
    b.close()
    assert {rid: len(t) for rid, t in b.outputs.items()} == {rid: len(t) for rid, t in a.outputs.items()}
    assert sb["steps"] > sa["steps"]                      # parallel threads shorten the critical path
    assert sb["peak_used_blocks"] >= sa["peak_used_blocks"]  # early release: never more cache than sequential
    # Sec. 3.4: per response, APAR never caches more tokens at once than sequential decoding holds at its end
    for r in reqs:
        assert a.infos[r.rid].max_cached_tokens <= flat[r.rid]
        assert a.infos[r.rid].attended_tokens <= b.infos[r.rid].attended_tokens
    pool.close()


def test_server_argument_checks():
    pool = ap.Pool(4, 2, 64, "f32", 16, dry_run=True)
    for bad in ((0, 0), (4, -1)):
        with pytest.raises(ap.AparError):
            ap.apar_server_create(pool.handle, *bad)
    srv = ap.apar_server_create(pool.handle, 2, 0)
    with pytest.raises(ap.AparError):
        ap.apar_server_submit(srv, 1, [])
    ap.apar_server_submit(srv, 7, list(range(20)))
    assert ap.apar_server_pop_finished(srv) is None
    assert ap.apar_server_admit(srv, None, None, 1 << 30) == (1, 20)
    b = ap.apar_server_batch(srv)
    assert len(b) == 1 and b["request_id"][0] == 7 and b["length"][0] == 20 and b["start_len"][0] == 20
    with pytest.raises(ap.AparError):
        ap.apar_server_step(srv, [1, 2], None, None)   # wrong batch size
    ap.apar_server_step(srv, [ap.APAR_TOKEN_EOS], None, None)
    rid, toks, info = ap.apar_server_pop_finished(srv)
    assert (rid, toks) == (7, [ap.APAR_TOKEN_EOS]) and info.generated_tokens == 1
    assert ap.apar_pool_stats(pool.handle).used_blocks == 0
    ap.apar_server_destroy(srv)
    pool.close()


def test_a_request_that_outgrows_the_pool_is_an_error_not_an_endless_replay():
    # one request whose response needs more blocks than the pool has: its prompt fits, so a policy that sent it
    # back to the queue would admit it again and replay the same overflow for ever.  The oldest running request
    # is never released; the step that does not fit returns OUT_OF_BLOCKS, in the library and in the oracle
    # alike, and leaves the books as they were.
    reqs = make_requests(1, seed=4, prompt_lo=40, prompt_hi=40)
    n_blocks = 4  # 64 token slots; the sampler writes at least 12 tokens per sequence and up to 260
    led = BlockLedger(n_blocks, max_threads=1 << 30)
    o = ServingOracle(led, 4, 0)
    pool = ap.Pool(4, 2, 64, "f32", n_blocks, max_threads=1 << 30, dry_run=True)
    srv = ap.apar_server_create(pool.handle, 4, 0)
    for r in reqs:
        o.submit(r.rid, r.prompt_tokens())
        ap.apar_server_submit(srv, r.rid, r.prompt_tokens())
    assert o.admit() == [0] and ap.apar_server_admit(srv, None, None, 1 << 30) == (1, 40)
    from oracle.ledger import OutOfBlocks

    for step in range(400):
        b = o.batch()
        lb = ap.apar_server_batch(srv)
        assert [e["thread"] for e in b] == lb["thread"].tolist() and b, "the request must still be running"
        xs = sample_tokens(CFG, [reqs[0].seed] * len(b), [e["seq_index"] for e in b], [e["length"] for e in b],
                           [e["last_token"] for e in b], [e["start_len"] for e in b], [e["group_size"] for e in b])
        # keep the response going: an [EOS] would let it finish before the pool is full
        xs = np.where(xs == ap.APAR_TOKEN_EOS, 5, xs).astype(np.int32)
        before = ap.apar_pool_stats(pool.handle)
        try:
            o.step(xs.tolist())
        except OutOfBlocks:
            with pytest.raises(ap.AparError) as e:
                ap.apar_server_step(srv, xs, None, None)
            assert e.value.status == -3
            after = ap.apar_pool_stats(pool.handle)
            assert (after.used_blocks, after.live_threads) == (before.used_blocks, before.live_threads)
            st = ap.apar_server_get_stats(srv)
            assert st.n_running == 1 and st.n_waiting == 0 and st.n_preemptions == 0
            assert len(o.running) == 1 and not o.waiting and o.preemptions == 0
            books_equal(pool.handle, led)
            break
        ap.apar_server_step(srv, xs, None, None)
        books_equal(pool.handle, led)
    else:
        raise AssertionError("the pool never filled up")
    ap.apar_server_destroy(srv)
    pool.close()
