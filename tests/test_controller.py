"""Algorithm 1 on top of the C ABI: pins for the plain-Python oracle, then the library's controller
against it on bookkeeping-only (dry-run) pools.  CPU only."""
import os

import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import TokenStream
from oracle import BlockLedger
from oracle.controller import CHILD, EOS, FORK, SequenceGroup

from harness import books_equal

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_restore_example.txt")
SYM = {"F": FORK, "E": EOS, "C": CHILD}


def _parse_golden():
    prompt, steps, want = [], [], {}
    for line in open(GOLDEN):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        vals = [SYM.get(x, None) if x in SYM else int(x) for x in f[1:]]
        if f[0] == "prompt":
            prompt = vals
        elif f[0] == "step":
            steps.append(vals)
        else:
            want[f[0]] = vals
    return prompt, steps, want


# -- oracle pins ---------------------------------------------------------------------------------
def test_oracle_worked_example():
    prompt, steps, want = _parse_golden()
    g = SequenceGroup(prompt)
    cached = []
    for s in steps:
        g.step(s)
        cached.append(g.cached_tokens())
    assert g.is_finished()
    assert g.restore() == want["restore"]
    assert g.attended == want["attended"][0] and g.generated == want["generated"][0]
    assert cached == want["cached"] and g.max_cached == want["max_cached"][0]


def test_oracle_without_forks_is_plain_decoding():
    g = SequenceGroup([7, 8])
    toks = [5, 6, 9, 4, EOS]
    for i, x in enumerate(toks):
        g.step([x])
        assert g.cached_tokens() == (0 if x == EOS else 2 + i + 1)
    assert g.restore() == toks
    assert g.attended == sum(2 + i for i in range(len(toks)))  # position of each token in the sequence
    assert g.max_cached == 2 + len(toks) - 1  # everything but the [EOS] step, when the cache is released


def _run_oracle_with_keys(seed, steps=120):
    """Drives the oracle with a seeded stream and labels every generated token with a key whose
    lexicographic order is the document order: a detail paragraph sorts right after the [Fork]
    that announced it and before what its parent generated next."""
    ts = TokenStream(seed, p_fork=0.08, p_eos=0.03, max_threads=9, max_len=90, min_len=25)
    g = SequenceGroup([1, 2, 3, 4])
    key_of = {0: [None] * 4}          # per sequence: key of each token (None for prompt / [Child])
    prefix = {0: ()}
    labelled = []
    for _ in range(steps):
        todo = g.unfinished()
        if not todo:
            break
        xs = ts.sample([s.last_token for s in todo], [len(s.tokens) for s in todo], len(g.G))
        before = len(g.G)
        forkers = [s for s in todo if s.last_token == FORK]
        g.step(xs)
        for s, c in zip(forkers, g.G[before:]):
            fork_key = key_of[s.sid][len(c.tokens) - 2]      # key of the [Fork] token that spawned c
            key_of[c.sid] = list(key_of[s.sid][: len(c.tokens) - 1]) + [None]
            prefix[c.sid] = fork_key + (0,)
        for s, x in zip(todo, xs):
            k = prefix[s.sid] + (len(s.tokens) - 1,)
            key_of[s.sid].append(k)
            labelled.append((k, x))
    return g, labelled


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_oracle_restore_is_document_order(seed):
    g, labelled = _run_oracle_with_keys(seed)
    assert len(g.G) > 2, "the stream should fork"
    want = [x for _, x in sorted(labelled, key=lambda kv: kv[0])]
    assert g.restore() == want
    assert len(want) == g.generated
    # Sec. 3.4: against the flattened (ordinary auto-regressive) output of the same length
    T, P = len(want), 4
    flat_attended = sum(P + i for i in range(T))
    assert g.attended < flat_attended
    assert g.max_cached <= P + T


# -- the library's controller against the oracle ------------------------------------------------------
def _drive_both(seed, n_blocks=4096, steps=200, **stream_kw):
    ts = TokenStream(seed, **stream_kw)
    rng = np.random.default_rng(seed)
    prompt = [int(x) for x in rng.integers(0, 1000, size=int(rng.integers(1, 40)))]
    pool = ap.Pool(4, 2, 64, "f32", n_blocks, dry_run=True)
    led = BlockLedger(n_blocks)
    grp = ap.apar_group_create(pool.handle, prompt, None, None)
    o = SequenceGroup(prompt)
    t0 = led.create()
    led.append(t0, len(prompt))
    tid = {0: t0}
    for step in range(steps):
        todo = o.unfinished()
        assert ap.apar_group_unfinished(grp) == [tid[s.sid] for s in todo]
        if not todo:
            break
        xs = ts.sample([s.last_token for s in todo], [len(s.tokens) for s in todo], len(o.G))
        forkers = [s for s in todo if s.last_token == FORK]
        before = len(o.G)
        rows = o.step(xs)
        info = ap.apar_group_step(grp, xs, None, None)
        for s, c in zip(forkers, o.G[before:]):
            (tid[c.sid],) = led.fork(tid[s.sid], 1)
        led.append_batch([tid[s.sid] for s in rows])
        for s, x in zip(todo, xs):
            if x == EOS:
                led.free(tid[s.sid])
        assert (info.n_forked, info.n_rows_appended) == (len(forkers), len(rows))
        assert info.n_finished == sum(1 for x in xs if x == EOS) and info.n_unfinished == len(o.unfinished())
        gi = ap.apar_group_get_info(grp)
        assert gi.cached_tokens == o.cached_tokens() and gi.max_cached_tokens == o.max_cached
        assert gi.attended_tokens == o.attended and gi.generated_tokens == o.generated
        assert gi.n_sequences == len(o.G)
        if step % 16 == 0:
            assert ap.apar_group_restore(grp) == o.restore()
            books_equal(pool.handle, led, check_blocks=range(0, n_blocks, 37))
    assert ap.apar_group_restore(grp) == o.restore()
    books_equal(pool.handle, led)
    return pool, grp, o, led


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5])
def test_controller_matches_oracle(seed):
    pool, grp, o, led = _drive_both(seed, p_fork=0.06, p_eos=0.02, max_threads=10, max_len=150, min_len=45)
    ap.apar_group_destroy(grp)
    st = ap.apar_pool_stats(pool.handle)
    assert st.live_threads == 0 and st.free_blocks == st.total_blocks  # destroy released what was left
    pool.close()


def test_golden_example_through_the_library():
    prompt, steps, want = _parse_golden()
    with ap.Pool(2, 2, 64, "f32", 16, dry_run=True) as pool:
        grp = ap.apar_group_create(pool.handle, prompt, None, None)
        cached = []
        for s in steps:
            ap.apar_group_step(grp, s, None, None)
            cached.append(ap.apar_group_get_info(grp).cached_tokens)
        assert cached == want["cached"]
        assert ap.apar_group_get_info(grp).max_cached_tokens == want["max_cached"][0]
        assert ap.apar_group_unfinished(grp) == []
        assert ap.apar_group_restore(grp) == want["restore"]
        gi = ap.apar_group_get_info(grp)
        assert gi.attended_tokens == want["attended"][0] and gi.generated_tokens == want["generated"][0]
        assert gi.n_sequences == 3 and gi.n_nodes == 5 and gi.cached_tokens == 0
        assert ap.apar_pool_stats(pool.handle).free_blocks == 16
        ap.apar_group_destroy(grp)


def test_step_that_does_not_fit_changes_nothing():
    with ap.Pool(2, 2, 64, "f32", 4, dry_run=True) as pool:  # 64 token slots
        grp = ap.apar_group_create(pool.handle, list(range(20)), None, None)   # blocks 0, 1
        ap.apar_group_step(grp, [FORK], None, None)              # root: 21 tokens
        ap.apar_group_step(grp, [5], None, None)                 # fork: the child copies the shared tail -> block 2
        assert ap.apar_pool_stats(pool.handle).free_blocks == 1
        for i in range(9):
            ap.apar_group_step(grp, [100 + i, 200 + i], None, None)
        ap.apar_group_step(grp, [FORK, 7], None, None)           # both sequences now hold 32 tokens: full tails
        snap = (ap.apar_group_restore(grp), ap.apar_group_unfinished(grp))
        st0 = ap.apar_pool_stats(pool.handle)
        with pytest.raises(ap.AparError) as ei:                  # a [Child] row and two rows at block boundaries
            ap.apar_group_step(grp, [3, 4], None, None)
        assert ei.value.status == -3
        st1 = ap.apar_pool_stats(pool.handle)
        assert (ap.apar_group_restore(grp), ap.apar_group_unfinished(grp)) == snap
        assert (st1.free_blocks, st1.live_threads, st1.cow_copies) == (st0.free_blocks, st0.live_threads, st0.cow_copies)
        assert st1.threads_issued == st0.threads_issued + 1      # ids are never reused, even after a rollback
        for b in range(4):
            assert ap.apar_block_refcount(pool.handle, b) == (2 if b == 0 else 1 if b < 3 else 0)
        with pytest.raises(ap.AparError):
            ap.apar_group_step(grp, [1], None, None)             # wrong count
        with pytest.raises(ap.AparError):
            ap.apar_group_step(grp, [CHILD, 1], None, None)      # [Child] is never sampled
        ap.apar_group_destroy(grp)
        assert ap.apar_pool_stats(pool.handle).free_blocks == 4
