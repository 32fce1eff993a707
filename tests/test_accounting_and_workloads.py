"""Closed-form pins for the token accounting, and checks of the seeded workload generator (CPU only)."""
import numpy as np
import pytest

from apar_workloads import (SpecLoopPlan, build_trace, draw_candidate_tree, make_config, mask_rows_from_parents,
                            node_kv, quantise, round_to_bf16_bits, bf16_bits_to_f32, step_q, tiny_tree)
from oracle import accounting as acc


def test_chain_equals_flatten():
    parents, segs = [-1, 0, 1, 2], [5, 7, 1, 16]
    T = sum(segs)
    assert acc.attended_tokens_tree(parents, segs) == acc.attended_tokens_flatten(parents, segs) == T * (T + 1) // 2
    assert acc.cached_tokens_shared(parents, segs) == acc.cached_tokens_copied(parents, segs) == T


@pytest.mark.parametrize("R,k,L", [(24, 3, 8), (100, 5, 40), (1, 2, 1)])
def test_star_closed_forms(R, k, L):
    parents, segs = [-1] + [0] * k, [R] + [L] * k
    T = R + k * L
    assert acc.attended_tokens_tree(parents, segs) == R * (R + 1) // 2 + k * (L * R + L * (L + 1) // 2)
    assert acc.attended_tokens_flatten(parents, segs) == T * (T + 1) // 2
    assert acc.cached_tokens_shared(parents, segs) == T
    assert acc.cached_tokens_copied(parents, segs) == k * (R + L)
    assert acc.path_lens(parents, segs)[1:] == [R + L] * k


def test_flatten_order_on_a_hand_worked_depth_two_tree():
    # Sec. 3.4 compares with the ordinary auto-regressive output of the same response, i.e. the paragraph tree
    # linearised in the order Alg. 1 restores it: a node, then its first child's subtree, then what followed.
    # Hand-worked, nodes in creation order (children created breadth first, so that depth-first and
    # breadth-first numbering disagree):
    #   0 root (5 tokens)  children 1, 2, 3
    #   1 (3 tokens)       children 4, 5        2 (2 tokens) no children        3 (4 tokens) child 6
    #   4 (7)   5 (1)   6 (6)
    # depth-first order of the nodes: 0 1 4 5 2 3 6, so the first tokens sit at
    #   0: 0   1: 5   4: 8   5: 15   2: 16   3: 18   6: 22      (total 28 tokens)
    # (breadth first would put node 2 at 8 and node 4 at 14).
    parents = [-1, 0, 0, 0, 1, 1, 3]
    segs = [5, 3, 2, 4, 7, 1, 6]
    assert acc.flatten_offsets(parents, segs) == [0, 5, 16, 18, 8, 15, 22]
    # attended tokens of the linearised sequence: token at position p (0-based) attends to p + 1 tokens
    assert acc.attended_tokens_flatten(parents, segs) == 28 * 29 // 2
    # in the tree a token sees its root path only: prefixes 0 / 5 5 5 / 8 8 / 9
    pre = [0, 5, 5, 5, 8, 8, 9]
    assert acc.prefix_lens(parents, segs) == pre
    # per node seg * prefix + seg (seg + 1) / 2:  15 + 21 + 13 + 30 + 84 + 9 + 75
    assert acc.attended_tokens_tree(parents, segs) == 247
    # a second tree after it starts again at 0
    assert acc.flatten_offsets(parents + [-1, 7], segs + [4, 2]) == [0, 5, 16, 18, 8, 15, 22, 0, 4]


def test_tree_never_attends_more_than_flatten():
    w = make_config("ht256", n_requests=12)
    parents = [n.parent for n in w.nodes]
    segs = [n.seg_len for n in w.nodes]
    off = acc.flatten_offsets(parents, segs)
    pre = acc.prefix_lens(parents, segs)
    assert all(p <= o for p, o in zip(pre, off))
    assert acc.attended_tokens_tree(parents, segs) < acc.attended_tokens_flatten(parents, segs)
    # sizes quoted in the byte report
    assert acc.kv_bytes(1, 32, 128, 2) == 16 * 1024 and acc.kv_bytes(1, 8, 128, 2) == 4 * 1024


def test_tiny_config_shape():
    w = tiny_tree()
    assert [n.seg_len for n in w.nodes] == [24, 8, 5, 12] and [n.parent for n in w.nodes] == [-1, 0, 0, 0]
    ops, live, nodes = build_trace(w)
    assert [o.kind for o in ops] == ["create", "append", "fork", "free", "append", "append", "append"]
    assert live == [1, 2, 3] and nodes == [1, 2, 3]
    assert [w.path_len(i) for i in w.leaves()] == [32, 29, 36]


@pytest.mark.parametrize("name", ["mha64", "ht256", "gqa1024", "spec128"])
def test_configs_are_seeded_and_prefix_stable(name):
    a = make_config(name, n_requests=6)
    b = make_config(name, n_requests=6)
    c = make_config(name, n_requests=9)
    sig = lambda w: [(n.request, n.parent, n.seg_len) for n in w.nodes]
    assert sig(a) == sig(b) == sig(c)[: len(a.nodes)]
    assert sig(make_config(name, seed=1, n_requests=6)) != sig(a)


def test_config_shapes_follow_the_recipe():
    w = make_config("mha64")
    roots = [n for n in w.nodes if n.parent < 0]
    assert len(roots) == 64 and all(256 + 64 <= n.seg_len <= 1024 + 64 for n in roots)
    assert all(4 <= len(n.children) <= 8 for n in roots)
    assert all(64 <= n.seg_len <= 256 for n in w.nodes if n.parent >= 0)
    assert max(n.depth for n in w.nodes) == 1
    w = make_config("ht256")
    roots = [n for n in w.nodes if n.parent < 0]
    assert len(roots) == 256 and all(2 <= len(n.children) <= 10 for n in roots)
    kids = [n for n in w.nodes if n.depth == 1]
    forked = [n for n in kids if n.children]
    assert 0.4 < len(forked) / len(kids) < 0.6 and all(2 <= len(n.children) <= 6 for n in forked)
    assert all(8 <= n.seg_len <= 512 for n in w.nodes if n.parent >= 0)
    assert max(n.depth for n in w.nodes) == 2
    assert 3000 < len(w.leaves()) < 4700  # about 3.8 k leaves expected
    assert w.heads.kv_bytes_per_token == 16384
    assert make_config("gqa1024", n_requests=2).heads.kv_bytes_per_token == 4096


def test_data_streams_are_per_node_and_bf16_exact():
    w = make_config("ht256", n_requests=2)
    k1, v1 = node_kv(w, 3)
    k2, v2 = node_kv(w, 3)
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2) and not np.array_equal(k1, v1)
    assert k1.shape == (w.nodes[3].seg_len, 32, 128) and k1.dtype == np.float32
    assert np.array_equal(quantise(k1, "bf16"), k1)  # already representable
    assert 0.06 < k1.std() < 0.12  # N(0,1)/sqrt(128)
    q = step_q(w, 0, 5)
    assert q.shape == (5, 32, 128) and not np.array_equal(q, step_q(w, 1, 5))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -1.0 - 2 ** -8, 3.14159], dtype=np.float32)
    got = bf16_bits_to_f32(round_to_bf16_bits(x))
    want = np.array([1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -1.0, 3.140625], dtype=np.float32)
    assert np.array_equal(got, want)
    import torch
    y = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    assert np.array_equal(bf16_bits_to_f32(round_to_bf16_bits(y)), torch.from_numpy(y).bfloat16().float().numpy())


def test_candidate_tree_masks():
    parents = np.array([-1, 0, 0, 2, 1])
    assert list(mask_rows_from_parents(parents)) == [0b00001, 0b00011, 0b00101, 0b01101, 0b10011]
    rng = np.random.default_rng(0)
    for _ in range(50):
        p = draw_candidate_tree(rng, 5)
        assert p[0] == -1 and all(0 <= p[c] < c for c in range(1, 5))
        m = mask_rows_from_parents(p)
        assert all((m[c] >> c) & 1 for c in range(5)) and all(m[c] < (1 << (c + 1)) for c in range(5))


def test_spec_loop_plan_is_consistent():
    plan = SpecLoopPlan(live=[3, 4, 7], next_tid=8, seed=0, p_fork=0.3, p_finish=0.2)
    live = {3, 4, 7}
    nxt = 8
    for _ in range(30):
        st = plan.next_step()
        assert st.live == sorted(live)
        assert set(st.finished) <= live and set(st.forked) <= live - set(st.finished)
        assert st.children == list(range(nxt, nxt + len(st.forked)))
        nxt += len(st.forked)
        for chain, par in zip(st.accepted, st.parents):
            assert chain[0] == 0 and all(par[b] == a for a, b in zip(chain[:-1], chain[1:]))
        live = (live - set(st.finished)) | set(st.children)
        if not live:
            break
    assert plan.live == sorted(live)
