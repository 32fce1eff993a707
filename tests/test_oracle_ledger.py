"""Pins for the bookkeeping half of the oracle (CPU only)."""
import itertools
import os

import numpy as np
import pytest

from apar_workloads import HeadConfig, build_trace, manual_tree, tiny_tree
from oracle import BlockLedger, DenseThreads, InvalidThread, OutOfBlocks

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tiny_ledger.txt")
B = 16


class TokenStore:
    """What the pool's memory would hold if rows were token ids: replays the ledger's
    writes and copies, so that reading a table back yields the tokens a thread can reach."""

    def __init__(self, n_blocks):
        self.slot = [[None] * B for _ in range(n_blocks)]

    def apply(self, ledger, token_ids):
        for src, dst, filled in ledger.last_copies:
            assert ledger.ref[dst] == 1
            self.slot[dst][:filled] = self.slot[src][:filled]
        assert len(ledger.last_writes) == len(token_ids)
        for (b, s), tok in zip(ledger.last_writes, token_ids):
            self.slot[b][s] = tok

    def read(self, ledger, t):
        L = ledger.len[t]
        return [self.slot[ledger.table[t][j // B]][j % B] for j in range(L)]


def replay(w, n_blocks, check_every_op=True):
    """Replay a workload's trace on the ledger and a token store; returns both plus bookkeeping."""
    ops, live, live_nodes = build_trace(w)
    led = BlockLedger(n_blocks)
    store = TokenStore(n_blocks)
    next_tok = 0
    toks_of_node = {}
    for op in ops:
        used, cows = led.used_blocks(), led.cow_copies
        if op.kind == "create":
            assert led.create() == op.tid
        elif op.kind == "append":
            toks = list(range(next_tok, next_tok + op.n_tokens))
            next_tok += op.n_tokens
            toks_of_node[op.node] = toks
            led.append(op.tid, op.n_tokens)
            assert len(led.last_copies) <= 1  # at most one block copied per thread per fork
            store.apply(led, toks)
        elif op.kind == "fork":
            assert tuple(led.fork(op.tid, len(op.children))) == op.children
            assert led.used_blocks() == used and led.cow_copies == cows  # a fork allocates and copies nothing
        elif op.kind == "free":
            led.free(op.tid)
        if check_every_op:
            led.check_invariants()
    return led, store, live, live_nodes, toks_of_node


def test_worked_example_matches_golden_file():
    led, _, live, _, _ = replay(tiny_tree(), 8)
    want = {"thread": {}, "refcount": {}}
    for line in open(GOLDEN):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "thread":
            want["thread"][int(f[1])] = (int(f[3]), [int(x) for x in f[5:]])
        elif f[0] == "refcount":
            want["refcount"][int(f[1])] = int(f[2])
        else:
            want[f[0]] = int(f[1])
    assert live == sorted(want["thread"])
    for t, (L, tab) in want["thread"].items():
        assert led.len[t] == L and led.table[t] == tab
    for b in range(8):
        assert led.ref[b] == want["refcount"].get(b, 0)
    assert led.used_blocks() == want["used_blocks"]
    assert led.cow_copies == want["cow_copies"]
    assert led.vanilla_blocks() == want["vanilla_blocks"]


def test_fork_shares_everything_and_refcount_counts_live_tables():
    led = BlockLedger(8)
    r = led.create()
    led.append(r, 24)
    kids = led.fork(r, 3)
    assert kids == [1, 2, 3]
    assert led.ref[:2] == [4, 4] and led.used_blocks() == 2
    assert all(led.table[k] == [0, 1] and led.len[k] == 24 for k in kids)
    led.free(r)
    assert led.ref[:2] == [3, 3]


def test_last_sharer_writes_in_place_and_full_tail_is_never_copied():
    led = BlockLedger(8)
    r = led.create()
    led.append(r, 32)  # two full blocks
    a, b = led.fork(r, 2)
    led.free(r)
    led.append(a, 1)
    led.append(b, 1)
    assert led.cow_copies == 0  # tail was full: nothing to copy
    assert led.table[a][:2] == [0, 1] and led.table[b][:2] == [0, 1]
    led2 = BlockLedger(8)
    r = led2.create()
    led2.append(r, 20)
    a, b = led2.fork(r, 2)
    led2.free(r)
    led2.append(a, 1)  # shared partial tail -> copy
    led2.append(b, 1)  # now the only holder -> in place
    assert led2.cow_copies == 1 and led2.table[b] == [0, 1] and led2.table[a] == [0, 2]


def test_free_order_and_lifo_reuse():
    led = BlockLedger(6)
    t = led.create()
    led.append(t, 40)  # blocks 0,1,2
    led.free(t)
    assert led.free_blocks() == 6
    u = led.create()
    led.append(u, 48)
    assert led.table[u] == [0, 1, 2]  # freed last-to-first, so they come back in table order
    led.check_invariants()


def test_out_of_blocks_is_transactional():
    led = BlockLedger(3)
    t = led.create()
    led.append(t, 20)
    snap = (list(led.ref), list(led.free_stack), dict(led.len), {k: list(v) for k, v in led.table.items()})
    with pytest.raises(OutOfBlocks):
        led.append(t, 40)
    assert snap == (led.ref, led.free_stack, led.len, led.table)
    a, = led.fork(t, 1)
    led.append(t, 1)  # copy-on-write takes the last block
    with pytest.raises(OutOfBlocks):
        led.append_batch([a, t, a] + [t] * 30)
    led.check_invariants()
    led.append(a, 1)  # sole holder now: in place, needs no block
    assert led.free_blocks() == 0


def test_invalid_thread():
    led = BlockLedger(4)
    t = led.create()
    led.free(t)
    for f in (lambda: led.append(t, 1), lambda: led.fork(t, 1), lambda: led.free(t)):
        with pytest.raises(InvalidThread):
            f()
    with pytest.raises(ValueError):
        led.fork(led.create(), 0)


def test_batch_append_equals_one_by_one_in_list_order():
    def build():
        led = BlockLedger(32)
        r = led.create()
        led.append(r, 21)
        kids = led.fork(r, 4)
        led.free(r)
        return led, kids

    a, kids = build()
    b, _ = build()
    order = [kids[2], kids[0], kids[3], kids[1], kids[2]]
    a.append_batch(order)
    for t in order:
        b.append(t, 1)
    assert a.table == b.table and a.ref == b.ref and a.free_stack == b.free_stack and a.cow_copies == b.cow_copies == 3


# -- brute force: every tree shape up to three levels with fan-out <= 3 ---------------
def _shapes(levels, max_fan=3):
    """All ordered trees with at most `levels` levels; a tree is the tuple of its children's trees."""
    if levels == 1:
        return [()]
    sub = _shapes(levels - 1, max_fan)
    out = [()]
    for k in range(1, max_fan + 1):
        out.extend(itertools.product(sub, repeat=k))
    return out


def _flatten_shape(shape):
    parents = []

    def rec(node, parent):
        idx = len(parents)
        parents.append(parent)
        for ch in node:
            rec(ch, idx)

    rec(shape, -1)
    return parents


SEG_CHOICES = (1, 15, 16, 17)
HEADS = HeadConfig(n_q_heads=2, n_kv_heads=1, head_dim=4, dtype="f32")


def test_all_tree_shapes_to_three_levels():
    shapes = _shapes(3)
    assert len(shapes) == 85
    rng = np.random.default_rng(0)
    n_checked = 0
    for shape in shapes:
        parents = _flatten_shape(shape)
        n = len(parents)
        for rot in range(4):
            segs = [SEG_CHOICES[(i + rot) % 4] for i in range(n)]
            w = manual_tree(parents, segs, HEADS)
            n_blocks = sum(-(-w.path_len(i) // B) for i in w.leaves()) + 2
            led, store, live, live_nodes, toks = replay(w, n_blocks)
            kids = {i: [c for c, p in enumerate(parents) if p == i] for i in range(n)}

            def leaves_below(i):
                return 1 if not kids[i] else sum(leaves_below(c) for c in kids[i])

            # the tokens reachable through a table are exactly the root path, in order
            for t, node in zip(live, live_nodes):
                expect = [x for a in w.root_path(node) for x in toks[a]]
                assert store.read(led, t) == expect
                assert len(led.table[t]) == -(-len(expect) // B)
            # refcount = number of live leaves that can reach the block
            seen = {}
            for t in live:
                for b in led.table[t]:
                    seen[b] = seen.get(b, 0) + 1
            assert all(led.ref[b] == seen.get(b, 0) for b in range(n_blocks))
            # a table slot lying wholly inside node a's own segment was popped fresh by a's
            # thread, so exactly the live leaves below a share it
            for t, node in zip(live, live_nodes):
                pos = 0
                for a in w.root_path(node):
                    for slot in range(-(-pos // B), (pos + segs[a]) // B):
                        assert led.ref[led.table[t][slot]] == leaves_below(a)
                    pos += segs[a]
            # vanilla layout and resident blocks
            assert led.vanilla_blocks() == sum(-(-w.path_len(i) // B) for i in w.leaves())
            assert led.used_blocks() <= led.vanilla_blocks()
            # free in every order (few leaves) or some seeded orders; nothing leaks
            orders = list(itertools.permutations(live)) if len(live) <= 4 else [list(rng.permutation(live)) for _ in range(3)]
            for order in orders[:24]:
                l2, _, _, _, _ = replay(w, n_blocks, check_every_op=False)
                for k, t in enumerate(order):
                    held_only_by_t = [b for b in l2.table[t] if l2.ref[b] == 1]
                    before = l2.free_blocks()
                    l2.free(t)
                    assert l2.free_blocks() - before == len(held_only_by_t)  # exactly the blocks only t held
                    l2.check_invariants()
                assert l2.free_blocks() == n_blocks and not l2.live()
            n_checked += 1
    assert n_checked == 85 * 4


def test_ledger_tokens_equal_dense_rows_on_random_traces():
    """Random interleavings of the five operations: the ledger plus a token store always
    reaches the same token sequence as the dense half's deep-copied rows."""
    rng = np.random.default_rng(1)
    for trial in range(40):
        n_blocks = 64
        led, store = BlockLedger(n_blocks), TokenStore(n_blocks)
        dense = DenseThreads(1, 1, 1)
        next_tok = 0
        t0 = led.create()
        assert dense.create() == t0
        for _ in range(60):
            live = led.live()
            if not live:
                break
            op = rng.choice(["append", "append", "fork", "free", "batch"])
            t = int(rng.choice(live))
            try:
                if op == "append":
                    n = int(rng.choice([1, 2, 15, 16, 17, 33]))
                    led.append(t, n)
                    toks = list(range(next_tok, next_tok + n))
                    next_tok += n
                    store.apply(led, toks)
                    dense.append(t, np.array(toks, float).reshape(n, 1, 1), np.zeros((n, 1, 1)))
                elif op == "batch":
                    ts = [int(x) for x in rng.choice(live, size=min(len(live), 3), replace=False)]
                    led.append_batch(ts)
                    toks = list(range(next_tok, next_tok + len(ts)))
                    next_tok += len(ts)
                    store.apply(led, toks)
                    for x, tok in zip(ts, toks):
                        dense.append(x, np.array([[[float(tok)]]]), np.zeros((1, 1, 1)))
                elif op == "fork":
                    n = int(rng.integers(1, 4))
                    assert led.fork(t, n) == dense.fork(t, n)
                elif len(live) > 1:
                    led.free(t)
                    dense.free(t)
            except OutOfBlocks:
                pass
            led.check_invariants()
            for x in led.live():
                assert store.read(led, x) == [int(v) for v in dense.rows(x)[0][:, 0, 0]]


def test_commit_candidates_books_equal_one_append_per_accepted_candidate():
    import copy

    led = BlockLedger(64)
    a = led.create()
    led.append(a, 21)
    kids = led.fork(a, 3)
    led.append(kids[0], 11)  # tail at slot 0 of a new block afterwards (21 + 11 = 32)
    one = copy.deepcopy(led)
    masks = [0b10110, 0b00000, 0b11111, 0b00001]
    led.commit_candidates([a] + kids, masks)
    for t, m in zip([a] + kids, masks):
        for _ in range(bin(m).count("1")):
            one.append(t, 1)
    assert led.table == one.table and led.len == one.len and led.ref == one.ref
    assert led.free_stack == one.free_stack and led.cow_copies == one.cow_copies
    assert [led.len[t] for t in [a] + kids] == [24, 32, 26, 22]
    led.check_invariants()
