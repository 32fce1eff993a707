"""Pins for the numeric half of the oracle (CPU only).

Each test fixes the oracle to something other than itself: a library routine on a
special case, a closed form, an invariant, or brute force on tiny inputs.
"""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import DenseThreads, attend, attend_spec


def _rng(seed):
    return np.random.default_rng(seed)


def _python_attend(q, K, V, scale):
    """Scalar-loop softmax attention in Python floats (fp64), no numpy linear algebra."""
    n_q, d = len(q), len(q[0])
    T, n_kv = len(K), len(K[0])
    g = n_q // n_kv
    out = [[0.0] * d for _ in range(n_q)]
    for h in range(n_q):
        kv = h // g
        s = []
        for j in range(T):
            acc = 0.0
            for x in range(d):
                acc += q[h][x] * K[j][kv][x]
            s.append(acc * scale)
        m = max(s)
        e = [math.exp(x - m) for x in s]
        z = sum(e)
        for j in range(T):
            for x in range(d):
                out[h][x] += (e[j] / z) * V[j][kv][x]
    return np.array(out)


# p1: a thread that never forks is ordinary causal decode attention ------------
@pytest.mark.parametrize("T,n_q,n_kv,d", [(1, 2, 2, 8), (17, 4, 4, 16), (40, 8, 2, 32)])
def test_no_fork_equals_causal_sdpa_last_row(T, n_q, n_kv, d):
    r = _rng(T)
    k = r.standard_normal((T, n_kv, d))
    v = r.standard_normal((T, n_kv, d))
    qs = r.standard_normal((T, n_q, d))  # a query for every position
    g = n_q // n_kv
    # library routine: causal self-attention over the whole sequence, fp64
    tq = torch.from_numpy(qs).permute(1, 0, 2)[None]  # [1, Hq, T, d]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(g, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(g, dim=0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0]  # [Hq, T, d]
    o = DenseThreads(n_q, n_kv, d)
    t = o.create()
    for j in range(T):
        o.append(t, k[j:j + 1], v[j:j + 1])  # append first, then decode (own row attended)
        out = o.decode(qs[j][None], [t])[0]
        np.testing.assert_allclose(out, ref[:, j, :].numpy(), rtol=0, atol=1e-12)


# brute force in scalar Python on tiny inputs --------------------------------
@pytest.mark.parametrize("T,n_q,n_kv,d", [(1, 1, 1, 1), (3, 2, 1, 2), (5, 4, 2, 3), (7, 6, 3, 2)])
def test_attend_matches_scalar_python(T, n_q, n_kv, d):
    r = _rng(100 + T)
    q = r.standard_normal((n_q, d))
    K = r.standard_normal((T, n_kv, d))
    V = r.standard_normal((T, n_kv, d))
    scale = 0.37
    np.testing.assert_allclose(attend(q, K, V, scale), _python_attend(q.tolist(), K.tolist(), V.tolist(), scale),
                               rtol=0, atol=1e-13)


# GQA head mapping: q head h must read kv head h // g ---------------------------
def test_gqa_head_mapping_revealed_by_values():
    n_q, n_kv, d, T = 8, 2, 4, 6
    r = _rng(5)
    K = r.standard_normal((T, n_kv, d))
    V = np.zeros((T, n_kv, d))
    for kv in range(n_kv):
        V[:, kv, :] = 10.0 + kv
    out = attend(r.standard_normal((n_q, d)), K, V, 0.5)
    for h in range(n_q):
        np.testing.assert_allclose(out[h], 10.0 + h // 4, atol=1e-12)


# p2: q = 0 gives the mean of V over exactly the root path ---------------------
def _build_tree_with_token_ids(o, parents, seg_lens, n_kv, d, rng):
    """Append rows whose V value is the token's global id; returns per-node thread id and id lists."""
    tid, ids, next_id = {}, {}, 0
    kids_of = {i: [c for c, p in enumerate(parents) if p == i] for i in range(len(parents))}
    order = []

    def visit(i):
        nonlocal next_id
        own = list(range(next_id, next_id + seg_lens[i]))
        next_id += seg_lens[i]
        ids[i] = (ids[parents[i]] if parents[i] >= 0 else []) + own
        if own:
            v = np.broadcast_to(np.array(own, dtype=np.float64)[:, None, None], (len(own), n_kv, d))
            o.append(tid[i], rng.standard_normal((len(own), n_kv, d)), v)
        if kids_of[i]:
            new = o.fork(tid[i], len(kids_of[i]))
            o.free(tid[i])
            for c, t in zip(kids_of[i], new):
                tid[c] = t
            for c in kids_of[i]:
                visit(c)
        else:
            order.append(i)

    for i, p in enumerate(parents):
        if p < 0:
            tid[i] = o.create()
            visit(i)
    return tid, ids, order


def test_zero_query_reveals_attended_token_set():
    n_q = n_kv = 2
    d = 4
    parents = [-1, 0, 0, 0, 2, 2, -1, 6]
    seg_lens = [24, 8, 5, 12, 1, 17, 3, 16]
    o = DenseThreads(n_q, n_kv, d)
    tid, ids, leaves = _build_tree_with_token_ids(o, parents, seg_lens, n_kv, d, _rng(0))
    threads = [tid[i] for i in leaves]
    out = o.decode(np.zeros((len(threads), n_q, d)), threads)
    for row, i in zip(out, leaves):
        np.testing.assert_allclose(row, np.mean(ids[i]), atol=1e-9)
        assert o.length(tid[i]) == len(ids[i])
    # second moment pins the exact multiset, not just its mean: V -> id^2
    o2 = DenseThreads(n_q, n_kv, d)
    t = o2.create()
    vals = np.array(ids[leaves[1]], dtype=np.float64)
    o2.append(t, np.zeros((len(vals), n_kv, d)), np.broadcast_to((vals ** 2)[:, None, None], (len(vals), n_kv, d)))
    np.testing.assert_allclose(o2.decode(np.zeros((1, n_q, d)), [t])[0], np.mean(vals ** 2), atol=1e-6)


# p3: one key with logit alpha, all others orthogonal -> closed form ---------------
@pytest.mark.parametrize("where", ["ancestor", "own"])
def test_peaked_closed_form(where):
    n_q = n_kv = 1
    d, alpha = 8, 40.0
    r = _rng(7)
    o = DenseThreads(n_q, n_kv, d)
    q = r.standard_normal(d)
    scale = o.scale

    def orth_rows(n):
        x = r.standard_normal((n, d))
        return x - np.outer(x @ q, q) / (q @ q)

    kstar = alpha * q / (scale * (q @ q))
    root = o.create()
    k_root, v_root = orth_rows(20), r.standard_normal((20, d))
    k_leaf, v_leaf = orth_rows(9), r.standard_normal((9, d))
    if where == "ancestor":
        k_root[3], star_v = kstar, v_root[3]
    else:
        k_leaf[5], star_v = kstar, v_leaf[5]
    o.append(root, k_root[:, None, :], v_root[:, None, :])
    a, b = o.fork(root, 2)
    o.free(root)
    o.append(a, k_leaf[:, None, :], v_leaf[:, None, :])
    o.append(b, orth_rows(4)[:, None, :], r.standard_normal((4, 1, d)))
    out = o.decode(q[None, None, :], [a])[0, 0]
    T = 29
    others = v_root.sum(0) + v_leaf.sum(0) - star_v
    expect = (math.exp(alpha) * star_v + others) / (math.exp(alpha) + T - 1)
    np.testing.assert_allclose(out, expect, rtol=0, atol=1e-9)
    np.testing.assert_allclose(out, star_v, atol=1e-12 + 40 * T * math.exp(-alpha))


# logits far beyond the range of exp: two keys a fixed distance apart, closed form ----
@pytest.mark.parametrize("level", [0.0, 2000.0, -2000.0, 1e5])
def test_two_keys_at_any_logit_level(level):
    """softmax is invariant under a shift of all logits: two keys whose logits are level and level + delta
    give weights 1 / (1 + e^delta) and e^delta / (1 + e^delta) whatever the level, also where e^level
    overflows or underflows a double."""
    d, delta = 4, 1.25
    q = np.array([[2.0, 0.0, 0.0, 0.0]])
    scale = 0.5
    # logit = scale * <q, k> = k[0]
    K = np.array([[[level, 3.0, -1.0, 0.5]], [[level + delta, -2.0, 4.0, 1.0]]])
    V = np.array([[[1.0, -2.0, 0.25, 8.0]], [[-3.0, 5.0, 0.5, -1.0]]])
    out = attend(q, K, V, scale)[0]
    w1 = math.exp(delta) / (1.0 + math.exp(delta))
    expect = (1.0 - w1) * V[0, 0] + w1 * V[1, 0]
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out, expect, rtol=0, atol=1e-9 * max(1.0, abs(level)) * 1e-3 + 1e-12)


# softmax shift invariance and the scale actually being applied -----------------
def test_scale_is_applied_and_default_is_inv_sqrt_d():
    r = _rng(11)
    q, K, V = r.standard_normal((2, 16)), r.standard_normal((5, 2, 16)), r.standard_normal((5, 2, 16))
    o = DenseThreads(2, 2, 16)
    assert o.scale == pytest.approx(0.25)
    t = o.create()
    o.append(t, K, V)
    np.testing.assert_allclose(o.decode(q[None], [t])[0], attend(q, K, V, 0.25), atol=0)
    # scaling q by c equals scaling the softmax scale by c
    np.testing.assert_allclose(attend(3.0 * q, K, V, 0.25), attend(q, K, V, 0.75), atol=1e-13)
    assert np.abs(attend(q, K, V, 0.25) - attend(q, K, V, 0.75)).max() > 1e-3


# p4: children of one fork see identical prefix logits -------------------------
def test_siblings_see_identical_prefix_logits():
    n_q, n_kv, d = 4, 2, 8
    r = _rng(3)
    o = DenseThreads(n_q, n_kv, d)
    root = o.create()
    o.append(root, r.standard_normal((21, n_kv, d)), r.standard_normal((21, n_kv, d)))
    kids = o.fork(root, 3)
    for k, n in zip(kids, (8, 5, 12)):
        o.append(k, r.standard_normal((n, n_kv, d)), r.standard_normal((n, n_kv, d)))
    q = r.standard_normal((n_q, d))
    base = o.logits(q, root)
    for k in kids:
        lg = o.logits(q, k)
        assert np.array_equal(lg[:, :21], base)  # bit-identical on the shared prefix
    # and a fork is a deep copy: growing one child leaves the parent and its siblings untouched
    assert o.length(root) == 21 and [o.length(k) for k in kids] == [29, 26, 33]


# p5: attention is a set operation over the root path ---------------------------
def test_order_invariance():
    r = _rng(9)
    q, K, V = r.standard_normal((3, 8)), r.standard_normal((33, 3, 8)), r.standard_normal((33, 3, 8))
    perm = r.permutation(33)
    np.testing.assert_allclose(attend(q, K, V, 0.3), attend(q, K[perm], V[perm], 0.3), atol=1e-14)


# p6: log-sum-exp merge of partial results over any split equals the whole --------
def test_merge_identity_every_split_point():
    r = _rng(21)
    T, d = 11, 4
    q, K, V = r.standard_normal((1, d)), 3 * r.standard_normal((T, 1, d)), r.standard_normal((T, 1, d))
    scale = 0.9
    whole = attend(q, K, V, scale)[0]

    def partial(lo, hi):
        s = scale * (K[lo:hi, 0] @ q[0])
        m = s.max()
        p = np.exp(s - m)
        return m, p.sum(), p @ V[lo:hi, 0]

    for cuts in itertools.chain(itertools.combinations(range(1, T), 1), itertools.combinations(range(1, T), 2)):
        edges = (0,) + cuts + (T,)
        parts = [partial(a, b) for a, b in zip(edges[:-1], edges[1:])]
        m = max(p[0] for p in parts)
        l = sum(p[1] * math.exp(p[0] - m) for p in parts)
        acc = sum(p[2] * math.exp(p[0] - m) for p in parts)
        np.testing.assert_allclose(acc / l, whole, atol=1e-13)


# p8: the multi-candidate step ----------------------------------------------------
def test_spec_single_candidate_equals_append_then_decode():
    n_q, n_kv, d = 4, 2, 8
    r = _rng(13)
    o = DenseThreads(n_q, n_kv, d)
    t = o.create()
    o.append(t, r.standard_normal((19, n_kv, d)), r.standard_normal((19, n_kv, d)))
    q = r.standard_normal((1, 1, n_q, d))
    ck, cv = r.standard_normal((1, 1, n_kv, d)), r.standard_normal((1, 1, n_kv, d))
    spec = o.decode_spec(q, ck, cv, np.array([[1]], dtype=np.uint8), [t])[0, 0]
    o.append(t, ck[0], cv[0])
    np.testing.assert_allclose(spec, o.decode(q[0], [t])[0], atol=1e-14)


def test_spec_chain_mask_equals_sequential_steps():
    n_q, n_kv, d, C = 2, 2, 4, 5
    r = _rng(17)
    o = DenseThreads(n_q, n_kv, d)
    t = o.create()
    o.append(t, r.standard_normal((7, n_kv, d)), r.standard_normal((7, n_kv, d)))
    q = r.standard_normal((1, C, n_q, d))
    ck, cv = r.standard_normal((1, C, n_kv, d)), r.standard_normal((1, C, n_kv, d))
    chain = np.array([[(1 << (c + 1)) - 1 for c in range(C)]], dtype=np.uint8)
    spec = o.decode_spec(q, ck, cv, chain, [t])[0]
    for c in range(C):
        o.append(t, ck[0, c:c + 1], cv[0, c:c + 1])
        np.testing.assert_allclose(spec[c], o.decode(q[0, c][None], [t])[0], atol=1e-14)


def test_spec_tree_mask_hides_other_branch():
    # candidates 1 and 2 are both children of 0: 2 must not see 1
    n_q = n_kv = 1
    d = 2
    K = np.zeros((1, 1, d))
    V = np.zeros((1, 1, d))
    ck = np.zeros((3, 1, d))
    cv = np.array([[[1.0, 0.0]], [[100.0, 0.0]], [[0.0, 1.0]]])
    masks = np.array([0b001, 0b011, 0b101], dtype=np.uint8)
    out = attend_spec(np.zeros((3, 1, d)), K, V, ck, cv, masks, 1.0)
    np.testing.assert_allclose(out[0, 0], [0.5, 0.0])  # cached row + itself
    np.testing.assert_allclose(out[1, 0], [101.0 / 3, 0.0])
    np.testing.assert_allclose(out[2, 0], [1.0 / 3, 1.0 / 3])  # no 100 from the other branch


def test_empty_thread_is_rejected():
    o = DenseThreads(1, 1, 2)
    t = o.create()
    with pytest.raises(ValueError):
        o.decode(np.zeros((1, 1, 2)), [t])


# commit of a multi-candidate step -------------------------------------------------
def test_commit_keeps_exactly_the_accepted_rows_in_candidate_order():
    # values reveal which rows were kept: candidate c of thread i carries the number 100*i + c
    n_kv, d, C = 1, 2, 5
    o = DenseThreads(1, n_kv, d)
    a, b = o.create(), o.create()
    o.append(a, np.full((3, n_kv, d), -1.0), np.full((3, n_kv, d), -1.0))
    o.append(b, np.full((1, n_kv, d), -2.0), np.full((1, n_kv, d), -2.0))
    ck = np.array([[[[100.0 * i + c] * d] for c in range(C)] for i in range(2)])
    cv = -ck
    o.commit_candidates([a, b], ck, cv, [0b01101, 0b00000])
    Ka, Va = o.rows(a)
    assert Ka[:, 0, 0].tolist() == [-1.0, -1.0, -1.0, 0.0, 2.0, 3.0] and Va[3:, 0, 1].tolist() == [-0.0, -2.0, -3.0]
    assert o.length(b) == 1  # nothing accepted: nothing changes
    # a thread listed twice gains both selections, in listed order
    o.commit_candidates([b, b], ck, cv, [0b10000, 0b00001])
    assert o.rows(b)[0][:, 0, 0].tolist() == [-2.0, 4.0, 100.0]


def test_commit_then_decode_equals_the_verified_candidate_row():
    # a chain of candidates, a prefix of it accepted: the decode output the accepted node's row got in
    # the multi-candidate step is the output of an ordinary decode after the commit
    n_q, n_kv, d, C = 2, 1, 4, 5
    r = _rng(23)
    o = DenseThreads(n_q, n_kv, d)
    t = o.create()
    o.append(t, r.standard_normal((9, n_kv, d)), r.standard_normal((9, n_kv, d)))
    q = r.standard_normal((1, C, n_q, d))
    ck, cv = r.standard_normal((1, C, n_kv, d)), r.standard_normal((1, C, n_kv, d))
    chain = np.array([[(1 << (c + 1)) - 1 for c in range(C)]], dtype=np.uint8)
    spec = o.decode_spec(q, ck, cv, chain, [t])[0]
    o.commit_candidates([t], ck, cv, [0b00111])
    assert o.length(t) == 12
    np.testing.assert_allclose(o.decode(q[0, 2][None], [t])[0], spec[2], atol=1e-14)


# prefill: the tree mask over whole segments -----------------------------------------
def test_prefill_of_an_unforked_thread_is_causal_sdpa():
    n_q, n_kv, d, T = 4, 2, 8, 37
    r = _rng(31)
    o = DenseThreads(n_q, n_kv, d)
    t = o.create()
    K, V = r.standard_normal((T, n_kv, d)), r.standard_normal((T, n_kv, d))
    o.append(t, K, V)
    q = r.standard_normal((T, n_q, d))
    got = o.prefill(q, [t], [T])
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]                          # [1, Hq, T, d]
    kt = torch.from_numpy(np.repeat(K, n_q // n_kv, axis=1)).permute(1, 0, 2)[None]
    vt = torch.from_numpy(np.repeat(V, n_q // n_kv, axis=1)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, atol=1e-12)
    # the last m queries only: the same rows of the full result
    np.testing.assert_allclose(o.prefill(q[-5:], [t], [5]), want[-5:], atol=1e-12)
    # m = 1 is the decode step
    np.testing.assert_allclose(o.prefill(q[-1:], [t], [1])[0], o.decode(q[-1:], [t])[0], atol=1e-14)


def test_prefill_of_a_tree_equals_sdpa_under_the_explicit_tree_mask():
    # nodes in creation order; every node's segment is prefetched as one thread.  The reference lays all
    # tokens of the tree side by side and masks token i -> token j by the definition: j's node is i's node
    # or an ancestor of it, and j comes no later than i where they share a node.
    parents = [-1, 0, 0, 1, 1, 2]
    seg = [5, 3, 4, 2, 6, 1]
    n_q, n_kv, d = 2, 1, 4
    r = _rng(37)
    o = DenseThreads(n_q, n_kv, d)
    tid = {}
    Kn = [r.standard_normal((s, n_kv, d)) for s in seg]
    Vn = [r.standard_normal((s, n_kv, d)) for s in seg]
    Qn = [r.standard_normal((s, n_q, d)) for s in seg]
    kids = {i: [j for j, p in enumerate(parents) if p == i] for i in range(len(parents))}
    order = []

    def visit(i):
        o.append(tid[i], Kn[i], Vn[i])
        order.append(i)
        if kids[i]:
            for j, t in zip(kids[i], o.fork(tid[i], len(kids[i]))):
                tid[j] = t
            for j in kids[i]:
                visit(j)

    tid[0] = o.create()
    visit(0)
    got = o.prefill(np.concatenate([Qn[i] for i in order]), [tid[i] for i in order], [seg[i] for i in order])
    # explicit mask over the concatenated tokens
    node_of = np.concatenate([[i] * seg[i] for i in order])
    pos_in = np.concatenate([np.arange(seg[i]) for i in order])
    anc = {i: set() for i in range(len(parents))}
    for i in range(len(parents)):
        a = parents[i]
        while a >= 0:
            anc[i].add(a)
            a = parents[a]
    N = len(node_of)
    mask = np.zeros((N, N), dtype=bool)
    for i in range(N):
        for j in range(N):
            mask[i, j] = (node_of[j] in anc[node_of[i]]) or (node_of[j] == node_of[i] and pos_in[j] <= pos_in[i])
    qt = torch.from_numpy(np.concatenate([Qn[i] for i in order])).permute(1, 0, 2)[None]
    kt = torch.from_numpy(np.repeat(np.concatenate([Kn[i] for i in order]), n_q, axis=1)).permute(1, 0, 2)[None]
    vt = torch.from_numpy(np.repeat(np.concatenate([Vn[i] for i in order]), n_q, axis=1)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=torch.from_numpy(mask))[0]
    np.testing.assert_allclose(got, want.permute(1, 0, 2).numpy(), atol=1e-12)
    # a sibling's tokens are invisible: changing node 1's values leaves node 2's rows alone
    assert not mask[node_of == 2][:, node_of == 1].any()


def test_prefill_rejects_bad_lengths():
    o = DenseThreads(1, 1, 2)
    t = o.create()
    o.append(t, np.ones((3, 1, 2)), np.ones((3, 1, 2)))
    for m in (0, 4):
        with pytest.raises(ValueError):
            o.prefill(np.ones((max(m, 1), 1, 2)), [t], [m])


# -- fp8 blocks: the rounding the oracle takes from torch, pinned to the format's definition ----------------
def _e4m3_values():
    """All finite values of OCP e4m3 from the definition: sign, 4 exponent bits (bias 7), 3 mantissa bits;
    exponent 0 is subnormal (mantissa / 8 * 2^-6); exponent 15 with mantissa 7 is NaN, everything else finite."""
    vals = []
    for e in range(16):
        for m in range(8):
            if e == 15 and m == 7:
                continue
            vals.append(m / 8 * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7))
    return np.array(sorted(set(vals)))


def test_fp8_rounding_is_round_to_nearest_even_on_the_e4m3_grid():
    from oracle import fp8

    grid = _e4m3_values()
    assert len(grid) == 127 and grid[0] == 0.0 and grid[-1] == 448.0 and grid[1] == 2.0 ** -9
    # every value of the format is a fixed point, both signs
    assert np.array_equal(fp8.round_e4m3(grid), grid) and np.array_equal(fp8.round_e4m3(-grid), -grid)
    # brute force: a dense sweep against "nearest grid value, ties to the one with an even mantissa"
    rng = np.random.default_rng(0)
    ys = np.concatenate([rng.uniform(-460, 460, 20000), rng.uniform(-1, 1, 20000), rng.uniform(-0.02, 0.02, 20000)])
    # the exact midpoints between neighbours are the ties
    mids = (grid[:-1] + grid[1:]) / 2
    ys = np.concatenate([ys, mids, -mids])
    ys = ys.astype(np.float32).astype(np.float64)   # what a float32 input holds
    got = fp8.round_e4m3(ys)
    idx = np.searchsorted(grid, np.abs(ys).clip(max=448.0))
    lo, hi = grid[np.maximum(idx - 1, 0)], grid[np.minimum(idx, len(grid) - 1)]
    a = np.abs(ys).clip(max=448.0)
    pick_hi = (hi - a < a - lo) | ((hi - a == a - lo) & (np.minimum(idx, len(grid) - 1) % 2 == 0))
    # (grid index parity = mantissa parity: index = 8 * exponent field + mantissa)
    want = np.sign(ys) * np.where(pick_hi, hi, lo)
    assert np.array_equal(got, want)


def test_fp8_tile_scale_and_lossless_grid():
    from apar_workloads import quantise
    from oracle import fp8

    assert fp8.tile_scale(np.zeros(4)) == 1.0
    for amax, s in ((448.0, 1.0), (448.5, 2.0), (224.0, 0.5), (224.1, 1.0), (1.0, 2.0 ** -8), (0.9, 2.0 ** -8), (0.875, 2.0 ** -9), (0.8, 2.0 ** -9),
                    (7.0, 2.0 ** -6), (3.6e-5, 2.0 ** -23)):
        assert fp8.tile_scale(np.array([0.0, -amax, amax / 3])) == s, amax
    # rows drawn for an fp8 pool sit on a grid that the tile rounding leaves alone, whatever rows share the tile
    rng = np.random.default_rng(1)
    for sigma in (1.0, 0.5, 1 / np.sqrt(128)):
        x = quantise((sigma * rng.standard_normal((64, 16, 128))).astype(np.float32), "bf16_fp8kv", kv=True)
        assert np.array_equal(quantise(x, "bf16"), x)          # bf16 can carry them to the library
        for tile in x:
            assert np.array_equal(fp8.sealed_tile(tile), tile.astype(np.float64))
        # also next to much larger or much smaller neighbours from the same grid
        mixed = x[0].copy()
        mixed[3] = quantise(np.full(128, 6.9, dtype=np.float32), "bf16_fp8kv", kv=True)
        assert np.array_equal(fp8.sealed_tile(mixed), mixed.astype(np.float64))
    # and plain bf16 data is NOT left alone (the test above would be vacuous otherwise)
    y = quantise(rng.standard_normal((16, 128)).astype(np.float32), "bf16")
    assert np.abs(fp8.sealed_tile(y) - y).max() > 1e-3
    K, V = fp8.cached_rows(np.tile(y[:, None, :], (3, 2, 1))[:40], np.tile(y[:, None, :], (3, 2, 1))[:40])
    assert np.array_equal(K[32:], np.tile(y[:, None, :], (3, 2, 1))[32:40]) and not np.array_equal(K[:16, 0], y)
