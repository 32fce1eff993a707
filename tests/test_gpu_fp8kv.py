"""Pools that keep full KV blocks in fp8 (APAR_BF16_FP8KV) against the oracle, through the C ABI (GPU only).

Two things are checked apart.  The quantiser: rows of arbitrary bf16 values go in, are read back, and must equal
oracle.fp8 (tile scale = smallest power of two that brings the tile under 448, e4m3 round to nearest even) bit
for bit, while rows of a block that is still filling come back untouched.  The attention path: inputs drawn on
the fp8 grid (which the library's rounding provably leaves alone, tests/test_oracle_numeric.py) are handed to the
library and to the dense oracle alike, and outputs are held to the bounds of the bf16 pools - the arithmetic
after the codes have been widened is the same."""
import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import (HeadConfig, draw_candidate_tree, make_config, manual_tree, mask_rows_from_parents,
                            node_kv_device, quantise, step_q)
from oracle import BlockLedger, DenseThreads, attend, fp8

from harness import (assert_close, blocks_upper_bound, books_equal, check_plan_covers_tables, nested_wide_tree,
                     pool_for, random_forest, replay_trace, to_dev, to_host)

pytestmark = pytest.mark.gpu
F8 = "bf16_fp8kv"


def torch():
    import torch as t

    return t


def decode_and_compare(w, pool, dense, live, step=0):
    t = torch()
    q = step_q(w, step, len(live))
    qd = to_dev(q, F8)
    out = t.full_like(qd, 9.0)
    ap.apar_decode_attention(pool.handle, qd, live, out)
    t.cuda.synchronize()
    return assert_close(to_host(out), dense.decode(q, live), F8, w.name)


def run(w, chunk=None, inline=True):
    N = blocks_upper_bound(w)
    hd = w.heads
    with pool_for(w, N) as pool:
        pool.kv.fill_(0xFF)
        if chunk:
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        ap.apar_set_inline_shared(pool.handle, inline)
        led = BlockLedger(N)
        dense = DenseThreads(hd.n_q_heads, hd.n_kv_heads, hd.head_dim)
        live, _ = replay_trace(w, pool, led, dense)
        books_equal(pool.handle, led)
        err = decode_and_compare(w, pool, dense, live)
        check_plan_covers_tables(pool.handle, live, hd.n_kv_heads, hd.n_q_heads // hd.n_kv_heads)
        info = ap.apar_last_plan_info(pool.handle)
        # bytes the call must move: full blocks at one byte per element plus two scales per (block, kv head),
        # blocks that are still filling at two bytes per element, queries in and outputs out
        held = {}
        for th in live:
            table, L = led.table[th], led.len[th]
            for i, b in enumerate(table):
                held[b] = min(16, L - 16 * i)
        full = sum(1 for v in held.values() if v == 16)
        open_tokens = sum(v for v in held.values() if v < 16)
        kv = 2 * hd.n_kv_heads * hd.head_dim
        assert info.algorithmic_bytes == full * (16 * kv + 8 * hd.n_kv_heads) + open_tokens * kv * 2 + \
            2 * len(live) * hd.n_q_heads * hd.head_dim * 2
        return err, info


def test_quantiser_matches_the_definition_bit_for_bit():
    """Arbitrary bf16 rows (several magnitudes, a tile of zeros, a huge outlier) in, cached rows out."""
    t = torch()
    heads = HeadConfig(4, 2, 128, F8)
    rng = np.random.default_rng(5)
    with ap.Pool(4, 2, 128, F8, 32) as pool:
        ap.apar_set_write_checks(pool.handle, True)
        pool.kv.fill_(0xFF)
        th = ap.apar_thread_create(pool.handle)
        L = 16 * 6 + 11
        scale = np.repeat(np.array([1.0, 0.01, 30.0, 0.0, 1e-6, 2.0, 1.0]), 16)[:L]
        K = quantise((rng.standard_normal((L, 2, 128)) * scale[:, None, None]).astype(np.float32), "bf16")
        V = quantise((rng.standard_normal((L, 2, 128)) * scale[::-1, None, None]).astype(np.float32), "bf16")
        K[37, 1, 5] = 6.0e4   # an outlier decides its tile's scale; its neighbours lose their low bits
        # appended in pieces that end inside blocks, at block ends and across them
        pos = 0
        for n in (5, 11, 1, 15, 16, 33, L - 81):
            ap.apar_append_kv(pool.handle, th, to_dev(K[pos:pos + n], F8), to_dev(V[pos:pos + n], F8))
            pos += n
        assert pos == L
        ko = t.empty((L, 2, 128), dtype=t.bfloat16, device="cuda:0")
        vo = t.empty_like(ko)
        ap.apar_read_kv_rows(pool.handle, th, 0, L, ko, vo)
        t.cuda.synchronize()
        Kw, Vw = fp8.cached_rows(K, V)
        assert np.array_equal(to_host(ko), Kw) and np.array_equal(to_host(vo), Vw)
        assert np.array_equal(Kw[96:], K[96:].astype(np.float64))        # the filling block: untouched
        assert not np.array_equal(Kw[:96], K[:96].astype(np.float64))    # full blocks: rounded
        # a fork shares the blocks; the child's copy-on-write copy of the filling block keeps its rows, and the
        # block is rounded once it fills up in the child
        (kid,) = ap.apar_fork(pool.handle, th, 1)
        extra = quantise(rng.standard_normal((7, 2, 128)).astype(np.float32), "bf16")
        ap.apar_append_kv(pool.handle, kid, to_dev(extra, F8), to_dev(extra, F8))
        ko2 = t.empty((L + 7, 2, 128), dtype=t.bfloat16, device="cuda:0")
        vo2 = t.empty_like(ko2)
        ap.apar_read_kv_rows(pool.handle, kid, 0, L + 7, ko2, vo2)
        ap.apar_read_kv_rows(pool.handle, th, 0, L, ko, vo)
        t.cuda.synchronize()
        Kc, Vc = fp8.cached_rows(np.concatenate([K, extra]), np.concatenate([V, extra]))
        assert np.array_equal(to_host(ko2), Kc) and np.array_equal(to_host(vo2), Vc)
        assert np.array_equal(to_host(ko), Kw) and np.array_equal(to_host(vo), Vw)  # the parent's rows did not move


def test_attention_over_rounded_blocks_equals_the_oracle_over_the_rounded_values():
    """Off-grid inputs: the oracle attends over oracle.fp8's values of the same rows."""
    t = torch()
    rng = np.random.default_rng(8)
    with ap.Pool(8, 2, 128, F8, 64) as pool:
        pool.kv.fill_(0xFF)
        th = ap.apar_thread_create(pool.handle)
        L = 16 * 9 + 6
        K = quantise(rng.standard_normal((L, 2, 128)).astype(np.float32), "bf16")
        V = quantise(rng.standard_normal((L, 2, 128)).astype(np.float32), "bf16")
        ap.apar_append_kv(pool.handle, th, to_dev(K, F8), to_dev(V, F8))
        q = quantise(rng.standard_normal((1, 8, 128)).astype(np.float32), "bf16")
        qd = to_dev(q, F8)
        out = t.empty_like(qd)
        ap.apar_decode_attention(pool.handle, qd, [th], out)
        t.cuda.synchronize()
        Kc, Vc = fp8.cached_rows(K, V)
        want = attend(q[0], Kc, Vc, 1.0 / np.sqrt(128.0))
        assert_close(to_host(out)[0], want, F8, "rounded blocks")
        # and the rounding matters at this tolerance: the oracle over the unrounded rows is further away
        plain = attend(q[0], K, V, 1.0 / np.sqrt(128.0))
        assert np.abs(plain - want).max() > 4 * np.abs(to_host(out)[0] - want).max()


@pytest.mark.parametrize("chunk", [1, 2, 8, None])
def test_ragged_trees_every_block_boundary(chunk):
    heads = HeadConfig(4, 4, 128, F8)
    parents = [-1, 0, 0, 0, 1, 1, 3, 3, 3, -1, -1, 10, 10]
    segs = [1, 15, 16, 17, 1, 33, 16, 15, 2, 1, 47, 1, 130]
    err, info = run(manual_tree(parents, segs, heads, seed=11), chunk=chunk)
    assert info.n_threads == 9


@pytest.mark.parametrize("g", [1, 4, 8])
def test_grouped_query_heads(g):
    heads = HeadConfig(8, 8 // g, 128, F8)
    run(manual_tree([-1, 0, 0, 0, 2, 2], [70, 9, 20, 33, 5, 18], heads, seed=2))


@pytest.mark.parametrize("name,n_req,scale", [("mha64", 4, None), ("mha64", 4, 1.0), ("ht256", 16, None),
                                              ("ht256", 6, 1.0), ("gqa1024", 2, None), ("gqa1024", 1, 1.0)])
def test_config_shaped_subsets(name, n_req, scale):
    w = make_config(name, n_requests=n_req, data_scale=scale, kv_fp8=True)
    err, info = run(w)
    print(f"{w.name} x{n_req} scale={scale}: max abs err {err:.3e}, {info.n_threads} threads")


@pytest.mark.parametrize("inline", [True, False])
@pytest.mark.parametrize("n_q,n_kv", [(2, 2), (8, 2)])
def test_wide_sharing_groups_cut_by_rank_or_standing_alone(n_q, n_kv, inline):
    w = nested_wide_tree(HeadConfig(n_q, n_kv, 128, F8), seed=6)
    err, info = run(w, inline=inline)
    assert (info.n_partial_rows == 0) == inline


@pytest.mark.parametrize("C,chunk", [(5, None), (3, 2), (8, None)])
def test_multi_candidate_step_and_commit(C, chunk):
    t = torch()
    heads = HeadConfig(4, 2, 128, F8)
    w = manual_tree([-1, 0, 0, 2, 2, -1], [30, 16, 9, 1, 25, 3], heads, seed=9, data_scale=0.7)
    N = blocks_upper_bound(w) + 8
    with pool_for(w, N) as pool:
        pool.kv.fill_(0xFF)
        if chunk:
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        led = BlockLedger(N)
        dense = DenseThreads(4, 2, 128)
        live, _ = replay_trace(w, pool, led, dense)
        n = len(live)
        rng = np.random.default_rng(1)
        for step in range(3):  # three steps: accepted candidates fill blocks up, which are then rounded
            q = quantise(0.7 * rng.standard_normal((n, C, 4, 128)).astype(np.float32), F8)
            ck = quantise(0.7 * rng.standard_normal((n, C, 2, 128)).astype(np.float32), F8, kv=True)
            cv = quantise(0.7 * rng.standard_normal((n, C, 2, 128)).astype(np.float32), F8, kv=True)
            masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, C)) for _ in range(n)])
            qd, ckd, cvd = to_dev(q, F8), to_dev(ck, F8), to_dev(cv, F8)
            out = t.empty_like(qd)
            ap.apar_decode_attention_spec(pool.handle, qd, ckd, cvd, t.from_numpy(masks).cuda(), C, live, out)
            t.cuda.synchronize()
            assert_close(to_host(out), dense.decode_spec(q, ck, cv, masks, live), F8, f"step {step}")
            accept = np.array([masks[i, int(rng.integers(0, C))] for i in range(n)], dtype=np.uint8)
            ap.apar_commit_candidates(pool.handle, live, ckd, cvd, C, accept)
            led.commit_candidates(live, accept)
            dense.commit_candidates(live, ck, cv, accept)
            books_equal(pool.handle, led)
        decode_and_compare(w, pool, dense, live, step=7)


@pytest.mark.parametrize("seed", range(6))
def test_random_forests_decode_spec_and_prefill(seed):
    t = torch()
    rng = np.random.default_rng(3000 + seed)
    n_kv = int(rng.choice([1, 2]))
    group = int(rng.choice([1, 2, 4, 8]))
    n_q = n_kv * group
    parents, segs = random_forest(rng, int(rng.integers(1, 4)), int(rng.integers(8, 120)))
    w = manual_tree(parents, segs, HeadConfig(n_q, n_kv, 128, F8), seed=seed, data_scale=0.5)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        pool.kv.fill_(0xFF)
        chunk = int(rng.choice([0, 1, 3, 7, 512]))
        if chunk:
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        ap.apar_set_matrix_units(pool.handle, int(rng.choice([0, 1, 64])), int(rng.choice([1, 2, 64])))  # ignored: no matrix units on fp8 pools
        ap.apar_set_inline_shared(pool.handle, bool(rng.integers(0, 2)))
        led = BlockLedger(N)
        dense = DenseThreads(n_q, n_kv, 128)
        live, nodes = replay_trace(w, pool, led, dense)
        books_equal(pool.handle, led)
        listed = [live[i] for i in rng.permutation(len(live))]
        decode_and_compare(w, pool, dense, listed, step=seed)
        wgs = np.array(ap.apar_last_plan_export(pool.handle, ap.APAR_PLAN_WORKGROUPS)).reshape(-1, 32)
        assert all(x & 255 in (1, 2) for x in wgs[:, 3]), "the 32x32 kernel reads bf16 tiles only"
        n = len(listed)
        C = int(rng.integers(1, 9))
        if C * group <= 64:
            q = quantise(0.5 * rng.standard_normal((n, C, n_q, 128)).astype(np.float32), F8)
            ck = quantise(0.5 * rng.standard_normal((n, C, n_kv, 128)).astype(np.float32), F8, kv=True)
            cv = quantise(0.5 * rng.standard_normal((n, C, n_kv, 128)).astype(np.float32), F8, kv=True)
            masks = np.stack([mask_rows_from_parents(draw_candidate_tree(rng, C)) for _ in range(n)])
            qd = to_dev(q, F8)
            out = t.empty_like(qd)
            ap.apar_decode_attention_spec(pool.handle, qd, to_dev(ck, F8), to_dev(cv, F8), t.from_numpy(masks).cuda(), C,
                                          listed, out)
            t.cuda.synchronize()
            assert_close(to_host(out), dense.decode_spec(q, ck, cv, masks, listed), F8, "candidates")
        m = [int(rng.integers(1, dense.length(th) + 1)) for th in listed]
        qp = quantise(0.5 * rng.standard_normal((sum(m), n_q, 128)).astype(np.float32), F8)
        qpd = to_dev(qp, F8)
        outp = t.empty_like(qpd)
        ap.apar_set_prefill_kernel(pool.handle, ap.APAR_PREFILL_MATRIX)  # the call stays on the row-tile kernel
        ap.apar_prefill_attention(pool.handle, qpd, listed, m, outp)
        t.cuda.synchronize()
        assert ap.apar_last_prefill_kernel(pool.handle) == ap.APAR_PREFILL_ROW_TILES
        assert_close(to_host(outp), dense.prefill(qp, listed, m), F8, "prefill")


def test_full_size_ht256_fp8_step_on_sampled_threads():
    """The headline workload on an fp8 pool through the benchmark's driver, N(0,1) data: sampled threads against
    the oracle over the very tensors the library was given (on the fp8 grid), and the bytes the plan reports."""
    t = torch()
    from paper_2401_06761_amd.driver import TreeRun

    w = make_config("ht256", data_scale=1.0, kv_fp8=True)
    hd = w.heads
    run_ = TreeRun(w, headroom_steps=8, churn=0.01)
    try:
        run_.build()
        for _ in range(2):
            run_.step(record=True)
        t.cuda.synchronize()
        out = run_.out.float().cpu().numpy().astype(np.float64)
        rec = run_.records[-1]
        live = rec.live
        rng = np.random.default_rng(0)
        sample = sorted(int(x) for x in rng.choice(len(live), size=16, replace=False))
        q_bank = run_.banks[rec.bank][0]
        wants = []
        for pos in sample:
            th = live[pos]
            ks, vs = [], []
            for a in w.root_path(run_.node_of[th]):
                k, v = node_kv_device(w, a)
                ks.append(k.float().cpu().numpy())
                vs.append(v.float().cpu().numpy())
            for bank, row in run_.extra_rows[th]:
                ks.append(run_.banks[bank][1][row:row + 1].float().cpu().numpy())
                vs.append(run_.banks[bank][2][row:row + 1].float().cpu().numpy())
            K, V = np.concatenate(ks).astype(np.float64), np.concatenate(vs).astype(np.float64)
            assert K.shape[0] == ap.apar_thread_len(run_.h, th)
            Kc, Vc = fp8.cached_rows(K, V)
            assert np.array_equal(Kc, K) and np.array_equal(Vc, V), "the driver's rows are on the grid the library keeps"
            wants.append(attend(q_bank[pos].float().cpu().numpy().astype(np.float64), K, V, 1.0 / np.sqrt(128.0)))
        worst = assert_close(out[sample], np.stack(wants), F8, "ht256 fp8")
        info = ap.apar_last_plan_info(run_.h)
        bf16_bytes = info.unique_tokens * 2 * 32 * 128 * 2
        assert 0.50 * bf16_bytes < info.algorithmic_bytes - 2 * len(live) * 32 * 128 * 2 < 0.56 * bf16_bytes
        print(f"ht256 on an fp8 pool: {len(live)} threads, sampled {len(sample)}, max abs err {worst:.2e}, "
              f"{info.algorithmic_bytes / 1e9:.2f} GB per call")
    finally:
        run_.close()
