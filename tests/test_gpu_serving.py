"""The serving loop on the GPU: real rows, decode attention over every step's batch against the dense
oracle, the scheduler's books against the oracle loop."""
import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import HeadConfig, SamplerConfig, make_requests, manual_tree, quantise, sample_tokens
from oracle import BlockLedger, DenseThreads
from oracle.serving import ServingOracle
from paper_2401_06761_amd.serving import ServingRun

from harness import books_equal, to_dev, to_host

pytestmark = pytest.mark.gpu
CFG = SamplerConfig(p_fork=0.06, p_eos=0.03, max_threads=6, min_new=10, max_len=140)


@pytest.mark.parametrize("n_blocks,max_running", [(2048, 8), (40, 6)])
def test_serving_loop_attention_and_books(n_blocks, max_running):
    import torch

    n_q, n_kv, d = 4, 2, 128
    reqs = make_requests(8, seed=5, prompt_lo=8, prompt_hi=60)
    rng = np.random.default_rng(0)
    R = 512
    qb = quantise(0.5 * rng.standard_normal((64, n_q, d)).astype(np.float32), "bf16")
    kb = quantise(0.5 * rng.standard_normal((R, n_kv, d)).astype(np.float32), "bf16")
    vb = quantise(0.5 * rng.standard_normal((R, n_kv, d)).astype(np.float32), "bf16")
    pool = ap.Pool(n_q, n_kv, d, "bf16", n_blocks, max_threads=1 << 20)
    pool.kv.fill_(0xFF)
    run = ServingRun(pool, reqs, CFG, max_running, 1, banks=(to_dev(qb, "bf16"), to_dev(kb, "bf16"), to_dev(vb, "bf16")))
    led = BlockLedger(n_blocks, max_threads=1 << 20)
    o = ServingOracle(led, max_running, 1)
    dense = DenseThreads(n_q, n_kv, d)
    by = {r.rid: r for r in reqs}
    for r in reqs:
        o.submit(r.rid, r.prompt_tokens())
    worst, steps = 0.0, 0
    while True:
        # the oracle's admission, mirrored row by row into the dense threads
        before = len(o.running)
        o.admit()
        used = 0
        for r in o.running[before:]:
            n = len(r["prompt"])
            while dense._next < r["tid"][0]:  # ids burnt by undone forks
                dense.free(dense.create())
            assert dense.create() == r["tid"][0]
            dense.append(r["tid"][0], kb[used:used + n], vb[used:used + n])
            used += n
        b = o.batch()
        more = run.step()
        if not b:
            assert not more
            break
        assert more
        torch.cuda.synchronize()
        threads = [e["thread"] for e in b]
        # (a request that the step preempted was still attended to before it: the batch is the pre-step one)
        got = to_host(run.out[:len(b)])
        want = dense.decode(qb[:len(b)], threads)
        worst = max(worst, float(np.abs(got - want).max()))
        xs = sample_tokens(CFG, [by[e["request_id"]].seed for e in b], [e["seq_index"] for e in b],
                           [e["length"] for e in b], [e["last_token"] for e in b], [e["start_len"] for e in b],
                           [e["group_size"] for e in b])
        n_before = [len(r["g"].unfinished()) + sum(s.last_token == -1 for s in r["g"].unfinished()) for r in o.running]
        victims = list(o.running)
        info = o.step(xs.tolist())
        row_ofs = np.concatenate([[0], np.cumsum(n_before)])
        for v in victims[len(victims) - info["n_preempted"]:]:
            for s in v["g"].unfinished():
                dense.free(v["tid"][s.sid])
        for p, c in info["forks"]:
            while dense._next < c:
                dense.free(dense.create())
            assert dense.fork(p, 1) == [c]
        for (ri, k), t in zip(info["rows"], info["row_threads"]):
            src = int(row_ofs[ri]) + k
            dense.append(t, kb[src:src + 1], vb[src:src + 1])
        for t in info["freed"]:
            dense.free(t)
        books_equal(pool.handle, led)
        steps += 1
    assert worst <= 2e-2, worst
    assert run.outputs == {rid: toks for rid, toks, _ in o.finished}
    st = ap.apar_server_get_stats(run.srv)
    assert st.n_preemptions == o.preemptions and (o.preemptions > 0) == (n_blocks < 100)
    print(f"serving loop: {steps} steps, {o.preemptions} preemptions, worst max abs err {worst:.2e}")
    run.close()
    pool.close()
