"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI (GPU only).

Tolerances (max abs error of attention outputs): 1e-5 for fp32 pools, 2e-2 for bf16 pools (bf16
inputs, fp32 accumulation, probabilities rounded to bf16 before the P.V product, bf16 output).
Block tables, lengths and refcounts are compared bit-exactly."""
import os

import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import (HeadConfig, make_config, manual_tree, mask_rows_from_parents, draw_candidate_tree,
                            node_kv, quantise, step_q, tiny_tree)
from oracle import BlockLedger, DenseThreads

from harness import assert_close, blocks_upper_bound, books_equal, check_plan_covers_tables, nested_wide_tree, pool_for, random_forest, replay_trace, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def torch():
    import torch as t

    return t


def poison(pool):
    """Fill the KV buffer with NaN bit patterns so that any read of an unwritten slot shows."""
    pool.kv.fill_(0xFF)


def decode_both(w, pool, dense, live, step=0, q=None):
    t = torch()
    hd = w.heads
    if q is None:
        q = step_q(w, step, len(live))
    qd = to_dev(q, hd.dtype)
    out = t.empty_like(qd)
    ap.apar_decode_attention(pool.handle, qd, live, out)
    t.cuda.synchronize()
    got = to_host(out)
    want = dense.decode(q, live)
    return got, want


def run_workload(w, chunk=None, check_each=False, sample=None, matrix_rows=None):
    N = blocks_upper_bound(w)
    hd = w.heads
    with pool_for(w, N) as pool:
        poison(pool)
        if chunk:
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        if matrix_rows is not None:
            ap.apar_set_matrix_units(pool.handle, matrix_rows, 1)
        led = BlockLedger(N)
        dense = DenseThreads(hd.n_q_heads, hd.n_kv_heads, hd.head_dim)
        live, nodes = replay_trace(w, pool, led, dense, check_each=check_each)
        books_equal(pool.handle, led)
        got, want = decode_both(w, pool, dense, live)
        err = assert_close(got, want, hd.dtype, w.name)
        info = ap.apar_last_plan_info(pool.handle)
        assert info.unique_blocks == led.used_blocks()
        return err, info


def test_tiny_fp32_tree_tables_and_attention():
    w = tiny_tree()
    with pool_for(w, 8) as pool:
        poison(pool)
        led = BlockLedger(8)
        dense = DenseThreads(2, 2, 64)
        live, _ = replay_trace(w, pool, led, dense, check_each=True)
        assert live == [1, 2, 3]
        assert [ap.apar_thread_block_table(pool.handle, t) for t in live] == [[0, 2], [0, 3], [0, 1, 4]]
        got, want = decode_both(w, pool, dense, live)
        assert np.abs(got - want).max() <= 1e-5
        st = ap.apar_pool_stats(pool.handle)
        assert st.bytes_resident == 5 * 16 * 1024 and st.bytes_vanilla == 7 * 16 * 1024


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 128)])
def test_rows_read_back_exactly_after_appends_forks_and_copies(dtype, d):
    t = torch()
    heads = HeadConfig(4, 2, d, dtype)
    w = manual_tree([-1, 0, 0, 1, 1, 2, -1, 6], [21, 3, 30, 1, 17, 16, 5, 40], heads, seed=3)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        led = BlockLedger(N)
        dense = DenseThreads(4, 2, d)
        live, _ = replay_trace(w, pool, led, dense, check_each=True)
        for th in live:
            L = dense.length(th)
            k = t.empty((L, 2, d), dtype=pool.torch_dtype, device="cuda:0")
            v = t.empty_like(k)
            ap.apar_read_kv_rows(pool.handle, th, 0, L, k, v)
            t.cuda.synchronize()
            K, V = dense.rows(th)
            assert np.array_equal(to_host(k), K) and np.array_equal(to_host(v), V)
        # one-row batch appends (with copy-on-write among siblings) land in the right slots too
        for step in range(3):
            k = quantise(np.random.default_rng(step).standard_normal((len(live), 2, d)).astype(np.float32), dtype)
            v = quantise(np.random.default_rng(100 + step).standard_normal((len(live), 2, d)).astype(np.float32), dtype)
            ap.apar_append_kv_batch(pool.handle, live, to_dev(k, dtype), to_dev(v, dtype))
            led.append_batch(live)
            for i, th in enumerate(live):
                dense.append(th, k[i:i + 1], v[i:i + 1])
        books_equal(pool.handle, led)
        for th in live:
            L = dense.length(th)
            k = t.empty((3, 2, d), dtype=pool.torch_dtype, device="cuda:0")
            v = t.empty_like(k)
            ap.apar_read_kv_rows(pool.handle, th, L - 3, 3, k, v)
            t.cuda.synchronize()
            K, V = dense.rows(th)
            assert np.array_equal(to_host(k), K[-3:]) and np.array_equal(to_host(v), V[-3:])


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 128)])
@pytest.mark.parametrize("chunk", [1, 2, 8])
def test_ragged_trees_every_block_boundary(dtype, d, chunk):
    heads = HeadConfig(4, 4, d, dtype)
    parents = [-1, 0, 0, 0, 1, 1, 3, 3, 3, -1, -1, 10, 10]
    segs = [1, 15, 16, 17, 1, 33, 16, 15, 2, 1, 47, 1, 130]
    w = manual_tree(parents, segs, heads, seed=11)
    err, info = run_workload(w, chunk=chunk, check_each=(chunk == 1))
    assert info.n_threads == 9


@pytest.mark.parametrize("g", [1, 4, 8])
def test_grouped_query_heads_bf16(g):
    heads = HeadConfig(8, 8 // g, 128, "bf16")
    w = manual_tree([-1, 0, 0, 0, 2, 2], [70, 9, 20, 33, 5, 18], heads, seed=2)
    run_workload(w)


def test_many_siblings_split_into_row_groups():
    # 70 children of one root: more than 64 rows share the root's blocks
    heads = HeadConfig(2, 2, 128, "bf16")
    parents = [-1] + [0] * 70
    segs = [100] + [1 + (i % 19) for i in range(70)]
    w = manual_tree(parents, segs, heads, seed=4)
    err, info = run_workload(w)
    assert info.n_threads == 70


@pytest.mark.parametrize("name,n_req,scale", [("mha64", 4, None), ("mha64", 4, 1.0), ("ht256", 16, None),
                                              ("ht256", 6, 1.0), ("gqa1024", 2, None), ("gqa1024", 1, 1.0)])
def test_config_shaped_subsets_bf16(name, n_req, scale):
    w = make_config(name, n_requests=n_req, data_scale=scale)
    err, info = run_workload(w)
    print(f"{name} x{n_req} scale={scale}: max abs err {err:.3e}, {info.n_threads} threads")


def test_zero_query_gives_mean_of_values_on_the_root_path():
    t = torch()
    heads = HeadConfig(2, 2, 128, "bf16")
    w = manual_tree([-1, 0, 0, 2, 2], [40, 13, 20, 7, 30], heads, seed=8)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        dense = DenseThreads(2, 2, 128)
        live, _ = replay_trace(w, pool, None, dense)
        q = np.zeros((len(live), 2, 128), dtype=np.float32)
        got, want = decode_both(w, pool, dense, live, q=q)
        for i, th in enumerate(live):
            mean = dense.rows(th)[1].mean(axis=0)
            assert np.abs(want[i] - mean).max() < 1e-12
            assert np.abs(got[i] - mean).max() <= 2e-3


def test_listed_threads_may_repeat_and_come_in_any_order():
    w = make_config("ht256", n_requests=3)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        dense = DenseThreads(32, 32, 128)
        live, _ = replay_trace(w, pool, None, dense)
        rng = np.random.default_rng(0)
        listed = [int(x) for x in rng.permutation(live)] + [live[0], live[0], live[-1]]
        got, want = decode_both(w, pool, dense, listed, step=3)
        assert np.abs(got - want).max() <= 2e-2
        one, want1 = decode_both(w, pool, dense, [live[2]], step=4)
        assert np.abs(one - want1).max() <= 2e-2


def test_parent_that_keeps_decoding_after_a_fork():
    # the paper's own shape (Alg. 1): the parent continues, a single child hangs off it
    t = torch()
    hd = HeadConfig(4, 4, 128, "bf16")
    w = manual_tree([-1], [0], hd, seed=6, data_scale=0.5)
    N = 64
    with pool_for(w, N) as pool:
        poison(pool)
        led = BlockLedger(N)
        dense = DenseThreads(4, 4, 128)
        rng = np.random.default_rng(6)

        def rows(n):
            return (quantise(0.5 * rng.standard_normal((n, 4, 128)).astype(np.float32), "bf16"),
                    quantise(0.5 * rng.standard_normal((n, 4, 128)).astype(np.float32), "bf16"))

        def append(th, n):
            k, v = rows(n)
            ap.apar_append_kv(pool.handle, th, to_dev(k, "bf16"), to_dev(v, "bf16"), n)
            led.append(th, n)
            dense.append(th, k, v)

        root = ap.apar_thread_create(pool.handle)
        assert led.create() == root == dense.create()
        append(root, 37)
        live = [root]
        for step in range(40):
            if step % 9 == 4:  # fork one child off the newest thread; both continue
                par = live[-1]
                kid = ap.apar_fork(pool.handle, par, 1)
                assert kid == led.fork(par, 1) == dense.fork(par, 1)
                live += kid
            for th in live:
                append(th, 1)
            books_equal(pool.handle, led)
            got, want = decode_both(w, pool, dense, live, step=step)
            assert np.abs(got - want).max() <= 2e-2
            if step == 30:  # early release of a finished thread while the rest go on
                gone = live.pop(1)
                ap.apar_free_thread(pool.handle, gone)
                led.free(gone)
                dense.free(gone)
        led.check_invariants()


@pytest.mark.parametrize("chunk", [None, 2])
@pytest.mark.parametrize("dtype,d,C", [("f32", 64, 5), ("f32", 128, 1), ("bf16", 128, 5), ("bf16", 128, 3),
                                       ("bf16", 128, 8)])
def test_multi_candidate_step(dtype, d, C, chunk):
    t = torch()
    heads = HeadConfig(4, 2, d, dtype)
    w = manual_tree([-1, 0, 0, 2, 2, -1], [30, 16, 9, 1, 25, 3], heads, seed=9, data_scale=0.7)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        if chunk:  # small units: partial results and the merge kernel fold the candidates instead
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        dense = DenseThreads(4, 2, d)
        live, _ = replay_trace(w, pool, None, dense)
        n = len(live)
        rng = np.random.default_rng(1)
        q = quantise(0.7 * rng.standard_normal((n, C, 4, d)).astype(np.float32), dtype)
        ck = quantise(0.7 * rng.standard_normal((n, C, 2, d)).astype(np.float32), dtype)
        cv = quantise(0.7 * rng.standard_normal((n, C, 2, d)).astype(np.float32), dtype)
        masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, C)) for _ in range(n)])
        qd = to_dev(q, dtype)
        out = t.empty_like(qd)
        ap.apar_decode_attention_spec(pool.handle, qd, to_dev(ck, dtype), to_dev(cv, dtype),
                                      t.from_numpy(masks).cuda(), C, live, out)
        t.cuda.synchronize()
        want = dense.decode_spec(q, ck, cv, masks, live)
        err = np.abs(to_host(out) - want).max()
        assert err <= TOL[dtype], err
        info = ap.apar_last_plan_info(pool.handle)
        e = heads.elem_bytes
        assert info.algorithmic_bytes == info.unique_tokens * heads.kv_bytes_per_token + \
            2 * n * C * 4 * d * e + 2 * n * C * 2 * d * e


def _fan_tree(fan, heads, seed):
    # a root of 40 tokens with `fan` children, every second child with two children of its own
    parents, lens = [-1], [40]
    for c in range(fan):
        parents.append(0)
        lens.append(5 + (c * 7) % 50)
        if c % 2:
            kid = len(parents) - 1
            parents += [kid, kid]
            lens += [3 + c % 20, 17]
    return manual_tree(parents, lens, heads, seed=seed, data_scale=0.5)


@pytest.mark.parametrize("dtype,n_q,n_kv,fan", [
    ("bf16", 2, 2, 40),    # 2 row tiles per wavefront
    ("bf16", 2, 2, 100),   # 4 row tiles per wavefront
    ("bf16", 2, 2, 150),   # more rows than one workgroup: stand-alone root, partial results
    ("bf16", 8, 1, 9),     # 8 rows per thread
    ("bf16", 8, 1, 20),
    ("f32", 2, 2, 100),
    ("f32", 8, 1, 20),
])
@pytest.mark.parametrize("chunk", [None, 3])
def test_wide_sharing_groups(dtype, n_q, n_kv, fan, chunk):
    w = _fan_tree(fan, HeadConfig(n_q, n_kv, 128, dtype), seed=fan)
    # stand-alone shared segments on the row-tile kernel, on the 32x32 kernel whenever they are wide, and by default
    for matrix_rows in ((0, 1, 64) if dtype == "bf16" else (None,)):
        err, info = run_workload(w, chunk=chunk, matrix_rows=matrix_rows)
        print(f"fan {fan}, matrix rows {matrix_rows}: {info.n_threads} threads, {info.n_partial_rows} partial rows, err {err:.2e}")


@pytest.mark.parametrize("n_cand", [1, 5])
def test_nested_wide_groups_inlined_stand_alone_and_matrix(n_cand):
    """A root with children that have more leaves than one unit carries, plus 200 threads listed right
    after their fork (they end at a shared segment): the plan inlines the short shared segments, or lets
    them stand alone (row-tile or matrix units), or mixes both; every variant against the oracle."""
    t = torch()
    heads = HeadConfig(2, 2, 128, "bf16")
    w = nested_wide_tree(heads, seed=9)
    N = blocks_upper_bound(w) + 600
    with pool_for(w, N) as pool:
        poison(pool)
        h = pool.handle
        dense = DenseThreads(2, 2, 128)
        live, _ = replay_trace(w, pool, None, dense)
        kids = ap.apar_fork(h, live[0], 200)
        assert dense.fork(live[0], 200) == kids
        listed = live + kids
        n = len(listed)
        rng = np.random.default_rng(4)
        q = quantise(0.5 * rng.standard_normal((n, n_cand, 2, 128)).astype(np.float32), "bf16")
        ck = quantise(0.5 * rng.standard_normal((n, n_cand, 2, 128)).astype(np.float32), "bf16")
        cv = quantise(0.5 * rng.standard_normal((n, n_cand, 2, 128)).astype(np.float32), "bf16")
        masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, n_cand)) for _ in range(n)])
        want = dense.decode_spec(q, ck, cv, masks, listed) if n_cand > 1 else dense.decode(q[:, 0], listed)[:, None]
        qd, ckd, cvd, md = to_dev(q, "bf16"), to_dev(ck, "bf16"), to_dev(cv, "bf16"), t.from_numpy(masks).cuda()
        seen_partials = set()
        for inline, matrix, chunk in ((True, (0, 0), 512), (False, (0, 0), 512), (True, (64, 8), 512), (True, (1, 1), 512),
                                      (True, (64, 8), 4), (False, (1, 1), 3), (True, (64, 16), 512)):
            ap.apar_set_inline_shared(h, inline)
            ap.apar_set_matrix_units(h, *matrix)
            ap.apar_set_chunk_blocks(h, chunk)
            out = t.empty_like(qd)
            if n_cand > 1:
                ap.apar_decode_attention_spec(h, qd, ckd, cvd, md, n_cand, listed, out)
            else:
                ap.apar_decode_attention(h, qd[:, 0].contiguous(), listed, out[:, 0])
            t.cuda.synchronize()
            got = to_host(out)
            err = np.abs(got - want).max()
            assert np.isfinite(got).all() and err <= TOL["bf16"], f"inline {inline} matrix {matrix} chunk {chunk}: {err}"
            seen_partials.add(ap.apar_last_plan_info(h).n_partial_rows)
        assert 0 in seen_partials and len(seen_partials) >= 4  # the variants really are different plans


@pytest.mark.parametrize("dtype,n_q,n_kv,d", [("bf16", 4, 2, 128), ("f32", 2, 2, 64)])
def test_long_threads_at_default_settings(dtype, n_q, n_kv, d):
    """Threads longer than the longest tile list one wavefront is given (512 blocks), with every knob at its
    default: a thread of 9000 tokens on its own, a shared segment of 8200 tokens below three threads, and a
    segment of 2100 tokens below 260 threads (wide and long enough for matrix units on a bf16 pool)."""
    t = torch()
    heads = HeadConfig(n_q, n_kv, d, dtype)
    parents, segs = [-1, -1, 1, 1, 1, -1], [9000, 8200, 1, 20, 600, 2100]
    for i in range(260):
        parents.append(5)
        segs.append(1 + i % 30)
    w = manual_tree(parents, segs, heads, seed=77, data_scale=0.5)
    with pool_for(w, blocks_upper_bound(w)) as pool:
        poison(pool)
        h = pool.handle
        dense = DenseThreads(n_q, n_kv, d)
        live, _ = replay_trace(w, pool, None, dense)
        n = len(live)
        rng = np.random.default_rng(6)
        q = quantise(0.5 * rng.standard_normal((n, 3, n_q, d)).astype(np.float32), dtype)
        ck = quantise(0.5 * rng.standard_normal((n, 3, n_kv, d)).astype(np.float32), dtype)
        cv = quantise(0.5 * rng.standard_normal((n, 3, n_kv, d)).astype(np.float32), dtype)
        masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, 3)) for _ in range(n)])
        qd, ckd, cvd, md = to_dev(q, dtype), to_dev(ck, dtype), to_dev(cv, dtype), t.from_numpy(masks).cuda()
        q1 = qd[:, 0].contiguous()
        out1, out = t.empty_like(q1), t.empty_like(qd)
        ap.apar_decode_attention(h, q1, live, out1)
        t.cuda.synchronize()
        info = ap.apar_last_plan_info(h)
        # all but the last child of a parent whose last block is open hold a copy of its filled slots
        assert info.n_partial_rows > 0 and info.unique_tokens == sum(segs) + 2 * (8200 % 16) + 259 * (2100 % 16)
        err = np.abs(to_host(out1) - dense.decode(q[:, 0], live)).max()
        assert err <= TOL[dtype], f"decode: {err}"
        check = check_plan_covers_tables(h, live, n_kv, rows_per_thread=n_q // n_kv)
        assert check["unit_block_reads"] >= check["unique_blocks"]
        ap.apar_decode_attention_spec(h, qd, ckd, cvd, md, 3, live, out)
        t.cuda.synchronize()
        err = np.abs(to_host(out) - dense.decode_spec(q, ck, cv, masks, live)).max()
        assert err <= TOL[dtype], f"three candidates: {err}"
        # prefill of the long threads' last tokens (their whole private tail where it is short)
        some = live[:4] + live[-2:]
        m = [min(dense.length(th), 40) for th in some]
        qp = quantise(0.5 * rng.standard_normal((sum(m), n_q, d)).astype(np.float32), dtype)
        qpd = to_dev(qp, dtype)
        outp = t.empty_like(qpd)
        ap.apar_prefill_attention(h, qpd, some, m, outp)
        t.cuda.synchronize()
        err = np.abs(to_host(outp) - dense.prefill(qp, some, m)).max()
        assert err <= TOL[dtype], f"prefill: {err}"


def _drift_direction(d):
    # 64 entries of +-1/8 (exact in bf16), norm 1
    u = np.zeros(d, dtype=np.float32)
    u[::2] = 0.125 * np.where(np.arange(d // 2) % 3 == 0, -1.0, 1.0)
    return u


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("mode", ["rising", "falling", "spread"])
def test_logits_far_from_the_running_reference(dtype, mode):
    """Softmax under stress.  rising: a token's logit grows by one bit per position, so every block of a
    path lifts the running maximum by sixteen bits (each unit rescales what it has summed at every tile, the
    partial results of a shared segment weigh nothing against the private ones).  falling: the mirror image
    (everything after a thread's first block underflows to probability zero, the shared root decides).
    spread: logits with a standard deviation of eleven bits.  Decode, multi-candidate and prefill calls, in
    every plan variant, against the oracle.

    fp32 pools are held to 1e-3 here rather than 1e-5: a dot product of magnitude 2600 carries an fp32
    rounding error of some 2e-3, i.e. 2e-4 in the logit and as much, relative, in a probability."""
    t = torch()
    tol = TOL["bf16"] if dtype == "bf16" else 1e-3
    heads = HeadConfig(2, 2, 128, dtype)
    w = nested_wide_tree(heads, seed=12)
    u = _drift_direction(128)
    slope = {"rising": 0.5, "falling": -0.5, "spread": 0.0}[mode]

    def kv_of(w_, node):
        k, v = node_kv(w_, node)
        start = w_.path_len(node) - w_.nodes[node].seg_len
        drift = slope * (start + np.arange(w_.nodes[node].seg_len, dtype=np.float32))
        return quantise(k + drift[:, None, None] * u, dtype), v

    def queries(rng, shape):
        noise = 0.5 * rng.standard_normal(shape).astype(np.float32)
        return quantise(32.0 * noise if mode == "spread" else 16.0 * u + noise, dtype)

    N = blocks_upper_bound(w) + 300
    with pool_for(w, N) as pool:
        poison(pool)
        h = pool.handle
        dense = DenseThreads(2, 2, 128)
        live, nodes = replay_trace(w, pool, None, dense, kv_of=kv_of)
        kids = ap.apar_fork(h, live[0], 100)
        assert dense.fork(live[0], 100) == kids
        listed = live + kids
        n = len(listed)
        rng = np.random.default_rng(31)
        for n_cand in (1, 5):
            q = queries(rng, (n, n_cand, 2, 128))
            # candidate keys continue the drift of their thread
            ck = 0.5 * rng.standard_normal((n, n_cand, 2, 128)).astype(np.float32)
            for i, th in enumerate(listed):
                ck[i] += slope * dense.length(th) * u
            ck = quantise(ck, dtype)
            cv = quantise(0.5 * rng.standard_normal((n, n_cand, 2, 128)).astype(np.float32), dtype)
            masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, n_cand)) for _ in range(n)])
            want = dense.decode_spec(q, ck, cv, masks, listed) if n_cand > 1 else dense.decode(q[:, 0], listed)[:, None]
            qd, ckd, cvd, md = to_dev(q, dtype), to_dev(ck, dtype), to_dev(cv, dtype), t.from_numpy(masks).cuda()
            for inline, matrix, chunk in ((True, (0, 0), 512), (False, (0, 0), 512), (True, (1, 1), 512), (False, (1, 1), 3)):
                ap.apar_set_inline_shared(h, inline)
                ap.apar_set_matrix_units(h, *matrix)
                ap.apar_set_chunk_blocks(h, chunk)
                out = t.empty_like(qd)
                if n_cand > 1:
                    ap.apar_decode_attention_spec(h, qd, ckd, cvd, md, n_cand, listed, out)
                else:
                    ap.apar_decode_attention(h, qd[:, 0].contiguous(), listed, out[:, 0])
                t.cuda.synchronize()
                got = to_host(out)
                err = np.abs(got - want).max()
                assert np.isfinite(got).all() and err <= tol, f"{n_cand} candidates, inline {inline} matrix {matrix} chunk {chunk}: {err}"
        # prefill over the last tokens of a few threads, both kernels on bf16 pools
        some = live[::40] + kids[:2]
        m = [min(dense.length(th), 50) for th in some]
        q = queries(rng, (sum(m), 2, 128))
        want = dense.prefill(q, some, m)
        qd = to_dev(q, dtype)
        for kernel in ([ap.APAR_PREFILL_ROW_TILES, ap.APAR_PREFILL_MATRIX] if dtype == "bf16" else [ap.APAR_PREFILL_AUTO]):
            ap.apar_set_prefill_kernel(h, kernel)
            out = t.empty_like(qd)
            ap.apar_prefill_attention(h, qd, some, m, out)
            t.cuda.synchronize()
            got = to_host(out)
            err = np.abs(got - want).max()
            assert np.isfinite(got).all() and err <= tol, f"prefill kernel {kernel}: {err}"


@pytest.mark.parametrize("dtype,fan,C,matrix_rows", [("bf16", 1, 5, 64), ("bf16", 3, 5, 64), ("bf16", 6, 5, 64), ("bf16", 6, 5, 1),
                                                     ("bf16", 40, 2, 64), ("bf16", 40, 2, 0), ("bf16", 11, 8, 64), ("bf16", 11, 8, 1),
                                                     ("f32", 3, 5, 64)])
def test_multi_candidate_wide_groups(dtype, fan, C, matrix_rows):
    t = torch()
    heads = HeadConfig(8, 1, 128, dtype)
    w = _fan_tree(fan, heads, seed=100 + fan)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        ap.apar_set_matrix_units(pool.handle, matrix_rows, 1)
        dense = DenseThreads(8, 1, 128)
        live, _ = replay_trace(w, pool, None, dense)
        n = len(live)
        rng = np.random.default_rng(fan)
        q = quantise(0.5 * rng.standard_normal((n, C, 8, 128)).astype(np.float32), dtype)
        ck = quantise(0.5 * rng.standard_normal((n, C, 1, 128)).astype(np.float32), dtype)
        cv = quantise(0.5 * rng.standard_normal((n, C, 1, 128)).astype(np.float32), dtype)
        masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, C)) for _ in range(n)])
        qd = to_dev(q, dtype)
        out = t.empty_like(qd)
        ap.apar_decode_attention_spec(pool.handle, qd, to_dev(ck, dtype), to_dev(cv, dtype),
                                      t.from_numpy(masks).cuda(), C, live, out)
        t.cuda.synchronize()
        want = dense.decode_spec(q, ck, cv, masks, live)
        got = to_host(out)
        assert np.isfinite(got).all()
        err = np.abs(got - want).max()
        assert err <= TOL[dtype], err


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_commit_candidates_rows_tables_and_next_decode(dtype, d):
    # several commit rounds over forked threads: rows cross block boundaries (blocks get sealed), shared
    # tails are copied on write; afterwards every row reads back exactly and a decode sees the new rows
    t = torch()
    heads = HeadConfig(4, 2, d, dtype)
    w = manual_tree([-1, 0, 0, 1, 1, 2, -1, 6], [21, 3, 30, 1, 17, 16, 5, 40], heads, seed=3, data_scale=0.5)
    N = blocks_upper_bound(w) + 32
    with pool_for(w, N) as pool:
        poison(pool)
        led = BlockLedger(N)
        dense = DenseThreads(4, 2, d)
        live, _ = replay_trace(w, pool, led, dense)
        rng = np.random.default_rng(77)
        for rnd, C in enumerate((5, 8, 1, 5, 5, 8)):
            n = len(live)
            ck = quantise(0.5 * rng.standard_normal((n, C, 2, d)).astype(np.float32), dtype)
            cv = quantise(0.5 * rng.standard_normal((n, C, 2, d)).astype(np.float32), dtype)
            masks = rng.integers(0, 1 << C, size=n).astype(np.uint8)
            if rnd == 1:
                masks[:] = (1 << C) - 1  # everything accepted
            if rnd == 2:
                masks[0] = 0
            ap.apar_commit_candidates(pool.handle, live, to_dev(ck, dtype), to_dev(cv, dtype), C, masks)
            led.commit_candidates(live, masks)
            dense.commit_candidates(live, ck, cv, masks)
            books_equal(pool.handle, led)
        for th in live:
            L = dense.length(th)
            k = t.empty((L, 2, d), dtype=pool.torch_dtype, device="cuda:0")
            v = t.empty_like(k)
            ap.apar_read_kv_rows(pool.handle, th, 0, L, k, v)
            t.cuda.synchronize()
            K, V = dense.rows(th)
            assert np.array_equal(to_host(k), K) and np.array_equal(to_host(v), V)
        got, want = decode_both(w, pool, dense, live, step=9)
        assert np.abs(got - want).max() <= TOL[dtype]
        led.check_invariants()


@pytest.mark.parametrize("dtype,n_q,n_kv,d", [("bf16", 4, 4, 128), ("bf16", 8, 2, 128), ("bf16", 8, 1, 128),
                                              ("bf16", 16, 1, 128), ("f32", 2, 2, 64), ("f32", 4, 1, 128)])
def test_prefill_attention_over_tree_segments(dtype, n_q, n_kv, d):
    t = torch()
    heads = HeadConfig(n_q, n_kv, d, dtype)
    parents = [-1, 0, 0, 1, 1, 2, -1, 6, 6]
    segs = [300, 15, 16, 17, 1, 33, 70, 130, 2]
    w = manual_tree(parents, segs, heads, seed=21, data_scale=0.5)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        dense = DenseThreads(n_q, n_kv, d)
        live, nodes = replay_trace(w, pool, None, dense)
        lens = [dense.length(th) for th in live]
        rng = np.random.default_rng(3)
        cases = [[w.nodes[i].seg_len for i in nodes], lens, [1] * len(live), [min(L, 20) for L in lens]]
        # bf16 pools have two prefill kernels; both are held to the oracle (fp32 pools have one)
        kernels = [ap.APAR_PREFILL_ROW_TILES, ap.APAR_PREFILL_MATRIX] if dtype == "bf16" else [ap.APAR_PREFILL_AUTO]
        for m in cases:
            q = quantise(0.5 * rng.standard_normal((sum(m), n_q, d)).astype(np.float32), dtype)
            qd = to_dev(q, dtype)
            want = dense.prefill(q, live, m)
            for kernel in kernels:
                ap.apar_set_prefill_kernel(pool.handle, kernel)
                out = t.empty_like(qd)
                ap.apar_prefill_attention(pool.handle, qd, live, m, out)
                t.cuda.synchronize()
                if dtype == "bf16":
                    assert ap.apar_last_prefill_kernel(pool.handle) == kernel
                got = to_host(out)
                assert np.isfinite(got).all()
                err = np.abs(got - want).max()
                assert err <= TOL[dtype], f"kernel {kernel}, m = {m}: max abs err {err}"
        ap.apar_set_prefill_kernel(pool.handle, ap.APAR_PREFILL_AUTO)
        # m = 1 is the decode step
        q = quantise(0.5 * rng.standard_normal((len(live), n_q, d)).astype(np.float32), dtype)
        qd = to_dev(q, dtype)
        a, b = t.empty_like(qd), t.empty_like(qd)
        ap.apar_prefill_attention(pool.handle, qd, live, [1] * len(live), a)
        ap.apar_decode_attention(pool.handle, qd, live, b)
        t.cuda.synchronize()
        assert np.abs(to_host(a) - to_host(b)).max() <= TOL[dtype]


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_append_kv_gather_takes_the_named_rows(dtype, d):
    t = torch()
    with ap.Pool(4, 2, d, dtype, 16) as pool:
        poison(pool)
        dense = DenseThreads(4, 2, d)
        a, b = ap.apar_thread_create(pool.handle), ap.apar_thread_create(pool.handle)
        assert (dense.create(), dense.create()) == (a, b)
        rng = np.random.default_rng(2)
        k = quantise(rng.standard_normal((40, 2, d)).astype(np.float32), dtype)
        v = quantise(rng.standard_normal((40, 2, d)).astype(np.float32), dtype)
        threads = [a, b, a, a, b] * 7
        src = [int(x) for x in rng.integers(0, 40, size=len(threads))]
        ap.apar_append_kv_gather(pool.handle, threads, src, to_dev(k, dtype), to_dev(v, dtype))
        for th, s_ in zip(threads, src):
            dense.append(th, k[s_:s_ + 1], v[s_:s_ + 1])
        for th in (a, b):
            L = dense.length(th)
            ko = t.empty((L, 2, d), dtype=pool.torch_dtype, device="cuda:0")
            vo = t.empty_like(ko)
            ap.apar_read_kv_rows(pool.handle, th, 0, L, ko, vo)
            t.cuda.synchronize()
            K, V = dense.rows(th)
            assert np.array_equal(to_host(ko), K) and np.array_equal(to_host(vo), V)


# APAR_TEST_FOREST_SEEDS / APAR_TEST_FOREST_NODES widen the sweep (more seeds, larger forests) for a one-off run
@pytest.mark.parametrize("seed", range(int(os.environ.get("APAR_TEST_FOREST_SEEDS", "10"))))
def test_random_forests_decode_spec_and_prefill(seed):
    """Seeded random forests (deep and wide mixes, segment lengths around the block boundaries), random head
    grouping, random unit caps: decode, multi-candidate decode and prefill against the dense oracle."""
    t = torch()
    rng = np.random.default_rng(1000 + seed)
    n_kv = int(rng.choice([1, 2]))
    group = int(rng.choice([1, 2, 4, 8]))
    n_q = n_kv * group
    heads = HeadConfig(n_q, n_kv, 128, "bf16")
    parents, segs = random_forest(rng, int(rng.integers(1, 4)),
                                  int(rng.integers(8, int(os.environ.get("APAR_TEST_FOREST_NODES", "120")))))
    w = manual_tree(parents, segs, heads, seed=seed, data_scale=0.5)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        poison(pool)
        chunk = int(rng.choice([0, 1, 3, 7, 512]))
        if chunk:
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        # stand-alone shared segments: never / always / by default on the 32x32 kernel
        ap.apar_set_matrix_units(pool.handle, int(rng.choice([0, 1, 64])), int(rng.choice([1, 2, 64])))
        ap.apar_set_inline_shared(pool.handle, bool(rng.integers(0, 2)))
        led = BlockLedger(N)
        dense = DenseThreads(n_q, n_kv, 128)
        live, nodes = replay_trace(w, pool, led, dense)
        books_equal(pool.handle, led)
        n = len(live)
        order = [int(x) for x in rng.permutation(n)]
        listed = [live[i] for i in order]
        got, want = decode_both(w, pool, dense, listed, step=seed)
        assert np.isfinite(got).all() and np.abs(got - want).max() <= TOL["bf16"]
        C = int(rng.integers(1, 9))
        q = quantise(0.5 * rng.standard_normal((n, C, n_q, 128)).astype(np.float32), "bf16")
        ck = quantise(0.5 * rng.standard_normal((n, C, n_kv, 128)).astype(np.float32), "bf16")
        cv = quantise(0.5 * rng.standard_normal((n, C, n_kv, 128)).astype(np.float32), "bf16")
        masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, C)) for _ in range(n)])
        if C * group <= 64:
            qd = to_dev(q, "bf16")
            out = t.empty_like(qd)
            ap.apar_decode_attention_spec(pool.handle, qd, to_dev(ck, "bf16"), to_dev(cv, "bf16"),
                                          t.from_numpy(masks).cuda(), C, listed, out)
            t.cuda.synchronize()
            wants = dense.decode_spec(q, ck, cv, masks, listed)
            gots = to_host(out)
            assert np.isfinite(gots).all() and np.abs(gots - wants).max() <= TOL["bf16"]
        m = [int(rng.integers(1, dense.length(th) + 1)) for th in listed]
        qp = quantise(0.5 * rng.standard_normal((sum(m), n_q, 128)).astype(np.float32), "bf16")
        qpd = to_dev(qp, "bf16")
        wantp = dense.prefill(qp, listed, m)
        for kernel in (ap.APAR_PREFILL_ROW_TILES, ap.APAR_PREFILL_MATRIX):
            ap.apar_set_prefill_kernel(pool.handle, kernel)
            outp = t.empty_like(qpd)
            ap.apar_prefill_attention(pool.handle, qpd, listed, m, outp)
            t.cuda.synchronize()
            assert ap.apar_last_prefill_kernel(pool.handle) == kernel
            gotp = to_host(outp)
            assert np.isfinite(gotp).all() and np.abs(gotp - wantp).max() <= TOL["bf16"], f"kernel {kernel}"
