"""Parity at the benchmark's full size, in the launch configuration bench.py times (GPU only).

The headline workload (256 requests, depth-2 fork trees, about 3.8 k live threads) is built and
stepped through the same driver bench.py uses.  The dense oracle cannot hold every thread's copy
of its rows in host memory, so attention outputs are compared on a seeded sample of threads
(whose rows are gathered from the very tensors handed to the library); block tables, refcounts
and counters are compared with the ledger for every thread; plan properties are checked whole.
"""
import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import build_trace, make_config, node_kv_device
from oracle import BlockLedger, attend
from paper_2401_06761_amd.driver import TreeRun

from harness import N_ID_BITS, assert_close, books_equal, id_channels

pytestmark = pytest.mark.gpu


def _replay_ledger(w, run, n_blocks):
    led = BlockLedger(n_blocks)
    ops, live, _ = build_trace(w)
    for op in ops:
        if op.kind == "create":
            led.create()
        elif op.kind == "append":
            led.append(op.tid, op.n_tokens)
        elif op.kind == "fork":
            led.fork(op.tid, len(op.children))
        else:
            led.free(op.tid)
    for rec in run.records:
        for pos, parent, child in rec.replaced:
            assert led.fork(parent, 1) == [child]
            led.free(parent)
        led.append_batch(rec.live)
    return led


# scale None: the configurations' own data, N(0,1)/sqrt(128) - a nearly uniform softmax with outputs of
# magnitude 0.02 at most; scale 1.0: N(0,1) data, whose logits spread the weights and whose outputs are large
# enough for the error bounds to bite.  gqa1024 runs whole once (1024 requests, a pool of about 60 GB).
@pytest.mark.parametrize("name,n_req,steps,scale", [("ht256", None, 3, None), ("ht256", None, 2, 1.0),
                                                    ("mha64", None, 2, None), ("mha64", None, 2, 1.0),
                                                    ("gqa1024", 48, 2, None), ("gqa1024", None, 1, 1.0)])
def test_full_size_step_matches_oracle_on_sampled_threads(name, n_req, steps, scale):
    import torch

    w = make_config(name, n_requests=n_req, data_scale=scale)
    hd = w.heads
    run = TreeRun(w, headroom_steps=steps + 4, churn=0.01)
    try:
        run.build()
        for _ in range(steps):
            run.step(record=True)
        torch.cuda.synchronize()
        out = run.out.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(out).all()
        rec = run.records[-1]
        live = rec.live
        # bookkeeping: every table, refcount and counter
        led = _replay_ledger(w, run, run.num_blocks)
        books_equal(run.h, led, check_blocks=range(0, run.num_blocks, 7))
        # plan: every block the live threads hold is read exactly once (MHA) and nothing else
        info = ap.apar_last_plan_info(run.h)
        st = ap.apar_pool_stats(run.h)
        assert info.unique_blocks == st.used_blocks == led.used_blocks()
        assert info.path_tokens == sum(led.len[t] for t in live)
        assert info.unique_tokens <= st.used_blocks * 16
        e = hd.elem_bytes
        assert info.algorithmic_bytes == info.unique_tokens * hd.kv_bytes_per_token + \
            2 * len(live) * hd.n_q_heads * hd.head_dim * e
        assert st.bytes_vanilla > 2 * st.bytes_resident  # prefix sharing pays off on these trees
        # attention: a seeded sample of threads, plus every thread a fork replaced in the last step
        rng = np.random.default_rng(0)
        sample = sorted(set(int(x) for x in rng.choice(len(live), size=20, replace=False)) |
                        set(pos for pos, _, _ in rec.replaced[:4]))
        q_bank = run.banks[rec.bank][0]
        wants = []
        for pos in sample:
            t = live[pos]
            node = run.node_of[t]
            ks, vs = [], []
            for a in w.root_path(node):
                k, v = node_kv_device(w, a)
                ks.append(k.float().cpu().numpy())
                vs.append(v.float().cpu().numpy())
            for bank, row in run.extra_rows[t]:
                ks.append(run.banks[bank][1][row:row + 1].float().cpu().numpy())
                vs.append(run.banks[bank][2][row:row + 1].float().cpu().numpy())
            K = np.concatenate(ks).astype(np.float64)
            V = np.concatenate(vs).astype(np.float64)
            assert K.shape[0] == ap.apar_thread_len(run.h, t)
            q = q_bank[pos].float().cpu().numpy().astype(np.float64)
            wants.append(attend(q, K, V, 1.0 / np.sqrt(hd.head_dim)))
        wants = np.stack(wants)
        worst = assert_close(out[sample], wants, hd.dtype, f"{name} scale {scale}")
        print(f"{name} scale {scale}: {len(live)} threads, sampled {len(sample)}, max abs err {worst:.2e}, "
              f"outputs up to {np.abs(wants).max():.3f}")
    finally:
        run.close()


def _id_rows_of(starts):
    """Rows whose values say where they come from: K is seeded noise (a zero query ignores it); V holds
    harness.id_channels of the token's global id (tokens numbered node by node) in every kv head, plus the
    bits of the kv head's index in dims 32..39 and their complements in 96..103."""
    def kv_of(w, node, device):
        import torch

        hd = w.heads
        n = w.nodes[node].seg_len
        k, _ = node_kv_device(w, node, device)
        vals = torch.from_numpy(id_channels(np.arange(starts[node], starts[node] + n))).to(device)
        v = vals[:, None, :].repeat(1, hd.n_kv_heads, 1)
        hbits = ((torch.arange(hd.n_kv_heads, device=device)[:, None] >> torch.arange(8, device=device)) & 1).float()
        v[:, :, 32:40] = hbits[None]
        v[:, :, 96:104] = 1.0 - hbits[None]
        return k, v.to(k.dtype)
    return kv_of


@pytest.mark.parametrize("name", ["ht256", "gqa1024"])
def test_full_size_zero_query_reveals_the_rows_read(name):
    """Which rows did the kernels read?  With a zero query the weights are uniform, so an output row is the
    mean of the V rows on its thread's root path; with values that encode each token's global id (and the kv
    head) that mean is fixed by the tree alone, and a block that is missing, foreign or read twice moves some
    channel by far more than bf16 rounding (tests/test_parity_bounds.py shows it on the CPU).  Runs at full
    size - pools of 12 GB and 60 GB, block offsets far beyond 2^32 - in the launch configuration of the
    benchmark; every thread is checked against the closed form and a sample against the oracle's attend()
    on the rows themselves."""
    import torch

    w = make_config(name)
    hd = w.heads
    starts = np.concatenate([[0], np.cumsum([n.seg_len for n in w.nodes])]).astype(np.int64)
    assert starts[-1] < 1 << N_ID_BITS
    kv_of = _id_rows_of(starts)
    run = TreeRun(w, headroom_steps=2, churn=0.0, kv_of=kv_of)
    try:
        run.build()
        live = run.live
        st = ap.apar_pool_stats(run.h)
        assert st.bytes_resident > 5 << 30, "the case is meant to reach block offsets beyond 2^32"
        top_block = max(ap.apar_thread_block_table(run.h, t)[-1] for t in live[-8:])
        assert top_block * st.block_bytes > 1 << 32
        q = torch.zeros((len(live), hd.n_q_heads, hd.head_dim), dtype=run.pool.torch_dtype, device="cuda:0")
        out = torch.full_like(q, 3.0)
        ap.apar_decode_attention(run.h, q, np.asarray(live, dtype=np.int32), out)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy().astype(np.float64)
        # closed form: per node the sum of its tokens' channels, per thread the sum along its root path
        node_sums = np.stack([id_channels(np.arange(starts[a], starts[a] + nd.seg_len)).astype(np.float64).sum(axis=0)
                              for a, nd in enumerate(w.nodes)])
        g = hd.n_q_heads // hd.n_kv_heads
        hb = (((np.arange(hd.n_q_heads)[:, None] // g) >> np.arange(8)) & 1).astype(np.float64)
        want = np.zeros((len(live), hd.n_q_heads, hd.head_dim))
        for i, t in enumerate(live):
            path = w.root_path(run.node_of[t])
            L = sum(w.nodes[a].seg_len for a in path)
            assert L == ap.apar_thread_len(run.h, t)
            want[i] = (node_sums[path].sum(axis=0) / L)[None, :]
            want[i, :, 32:40] = hb
            want[i, :, 96:104] = 1.0 - hb
        # sums of these values are exact in fp32, so all that separates got from want is one rounding to bf16
        excess = np.abs(got - want) - (2.0 ** -8 * np.abs(want) + 1e-6)
        assert excess.max() <= 0, f"thread at list position {int(excess.max(axis=(1, 2)).argmax())}: off by {excess.max()}"
        # the oracle on the rows themselves, for a sample
        rng = np.random.default_rng(3)
        for pos in sorted(int(x) for x in rng.choice(len(live), size=8, replace=False)):
            ks, vs = zip(*[kv_of(w, a, "cuda:0") for a in w.root_path(run.node_of[live[pos]])])
            K = torch.cat(ks).float().cpu().numpy().astype(np.float64)
            V = torch.cat(vs).float().cpu().numpy().astype(np.float64)
            ref = attend(np.zeros((hd.n_q_heads, hd.head_dim)), K, V, 1.0 / np.sqrt(hd.head_dim))
            assert np.abs(ref - want[pos]).max() < 1e-12
        print(f"{name}: {len(live)} threads, {st.bytes_resident / 2**30:.1f} GiB resident, highest block offset "
              f"{top_block * st.block_bytes / 2**30:.1f} GiB, worst deviation from the path mean "
              f"{np.abs(got - want).max():.2e}")
    finally:
        run.close()


@pytest.mark.parametrize("scale", [None, 1.0])
def test_full_size_speculative_loop_on_sampled_threads(scale):
    """The 256-step multi-candidate loop on all 128 requests of spec128, as bench.py runs it (fixed candidate
    bank, accepted rows committed from the candidate arrays): the ledger follows every operation; counters
    and the tables of a fixed sample of threads are compared after every step, all tables and refcounts at
    steps 0, 1, 2, 64, 128 and 255; at those steps the attention outputs of threads of four requests are
    compared with the dense oracle, whose rows are gathered from the tensors handed to the library along the
    history of each thread (tree nodes, accepted candidate rows, the row a forked child received)."""
    import torch

    from oracle import attend_spec
    from paper_2401_06761_amd.driver import SpecRun

    n_steps, C = 256, 5
    check_steps = {0, 1, 2, 64, 128, 255}
    w = make_config("spec128", data_scale=scale)
    hd = w.heads
    sm_scale = 1.0 / np.sqrt(hd.head_dim)
    run = SpecRun(w, n_steps, n_cand=C)
    try:
        run.build()
        h = run.h
        N = run.peak_blocks + 64
        led = BlockLedger(N)
        ops, live, live_nodes = build_trace(w)
        for op in ops:
            if op.kind == "create":
                led.create()
            elif op.kind == "append":
                led.append(op.tid, op.n_tokens)
            elif op.kind == "fork":
                led.fork(op.tid, len(op.children))
            else:
                led.free(op.tid)
        books_equal(h, led, check_blocks=range(0, N, 97))
        tracked_requests = {0, 17, 64, 127}
        hist = {t: [("node", a) for a in w.root_path(nd)] for t, nd in zip(live, live_nodes)
                if w.nodes[nd].request in tracked_requests}
        node_rows = {}

        def rows_of(t, bank_k, bank_v, child_k, child_v):
            ks, vs = [], []
            for item in hist[t]:
                if item[0] == "node":
                    if item[1] not in node_rows:
                        k, v = node_kv_device(w, item[1])
                        node_rows[item[1]] = (k.float().cpu().numpy(), v.float().cpu().numpy())
                    k, v = node_rows[item[1]]
                elif item[0] == "cand":
                    k = bank_k[item[1], item[2]][None].float().cpu().numpy()
                    v = bank_v[item[1], item[2]][None].float().cpu().numpy()
                else:
                    k = child_k[item[1]][None].float().cpu().numpy()
                    v = child_v[item[1]][None].float().cpu().numpy()
                ks.append(k), vs.append(v)
            return np.concatenate(ks).astype(np.float64), np.concatenate(vs).astype(np.float64)

        rng = np.random.default_rng(1)
        watch = [int(t) for t in rng.choice(live, size=24, replace=False)]  # tables checked after every step
        worst, n_checked, peak = 0.0, 0, led.used_blocks()
        bank_q, bank_k, bank_v = run.bank
        child_k, child_v = run.child_bank
        for s in range(n_steps):
            st, q, ck, cv, out, kk, vv = run.step()
            if s in check_steps:
                torch.cuda.synchronize()
                pos_of = {t: i for i, t in enumerate(st.live)}
                mine = [t for t in st.live if t in hist]
                pick = [int(t) for t in rng.choice(mine, size=min(10, len(mine)), replace=False)]
                for t in pick:
                    i = pos_of[t]
                    K, V = rows_of(t, bank_k, bank_v, child_k, child_v)
                    assert K.shape[0] == led.len[t]
                    want = attend_spec(q[i].float().cpu().numpy().astype(np.float64), K, V,
                                       ck[i].float().cpu().numpy().astype(np.float64),
                                       cv[i].float().cpu().numpy().astype(np.float64), st.masks[i], sm_scale)
                    got = out[i].float().cpu().numpy().astype(np.float64)
                    worst = max(worst, assert_close(got, want, hd.dtype, f"step {s}, thread {t}"))
                    n_checked += 1
            # the same bookkeeping on the oracle side
            led.commit_candidates(st.live, st.accept_masks)
            peak = max(peak, led.used_blocks())
            for i, t in enumerate(st.live):
                if t in hist:
                    hist[t] += [("cand", i, c) for c in range(C) if st.accept_bits[i, c]]
            for t in st.finished:
                led.free(t)
                hist.pop(t, None)
            for m, (t, child) in enumerate(zip(st.forked, st.children)):
                assert led.fork(t, 1) == [child]
                if t in hist:
                    hist[child] = hist[t] + [("child", m)]
                if t in watch and len(watch) < 48:
                    watch.append(child)
            if st.children:
                led.append_batch(st.children)
            peak = max(peak, led.used_blocks())
            stats = ap.apar_pool_stats(h)
            assert stats.used_blocks == led.used_blocks() and stats.live_threads == len(run.live)
            assert stats.cow_copies == led.cow_copies and stats.threads_issued == led.next_tid
            watch = [t for t in watch if t in led.table]
            for t in watch:
                assert ap.apar_thread_len(h, t) == led.len[t] and ap.apar_thread_block_table(h, t) == led.table[t]
            if s in check_steps:
                books_equal(h, led, check_blocks=range(0, N, 97))
                assert sorted(run.live) == led.live()
        led.check_invariants()
        assert peak == run.peak_blocks and n_checked >= 50
        print(f"spec128 loop (data scale {scale}), 128 requests x {n_steps} steps: {len(run.live)} live threads at the end, "
              f"{n_checked} sampled outputs, worst max abs err {worst:.2e}, peak {peak} blocks")
    finally:
        run.close()
