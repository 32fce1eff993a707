"""Algorithm 1 end to end on the GPU: several sequence groups decode together, the controller forks,
appends and releases through the ABI, and every step's attention is checked against the dense oracle."""
import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import TokenStream, quantise
from oracle import DenseThreads
from oracle.controller import EOS, FORK, SequenceGroup

from harness import to_dev, to_host

pytestmark = pytest.mark.gpu


def test_groups_decode_with_forks_and_early_release():
    import torch

    n_q, n_kv, d, dtype = 4, 2, 128, "bf16"
    rng = np.random.default_rng(3)

    def rows(n):
        return (quantise(0.6 * rng.standard_normal((n, n_kv, d)).astype(np.float32), dtype),
                quantise(0.6 * rng.standard_normal((n, n_kv, d)).astype(np.float32), dtype))

    with ap.Pool(n_q, n_kv, d, dtype, 512) as pool:
        pool.kv.fill_(0xFF)
        dense = DenseThreads(n_q, n_kv, d)
        groups = []
        for gi in range(5):
            prompt = [int(x) for x in rng.integers(0, 100, size=int(rng.integers(3, 50)))]
            k, v = rows(len(prompt))
            grp = ap.apar_group_create(pool.handle, prompt, to_dev(k, dtype), to_dev(v, dtype))
            o = SequenceGroup(prompt)
            tid = {0: ap.apar_group_unfinished(grp)[0]}
            assert dense.create() == tid[0]
            dense.append(tid[0], k, v)
            groups.append((grp, o, tid, TokenStream(gi, p_fork=0.07, p_eos=0.02, max_threads=8, max_len=110,
                                                    min_len=30)))
        worst, steps, max_live = 0.0, 0, 0
        while any(not o.is_finished() for _, o, _, _ in groups) and steps < 140:
            live = [t for grp, _, _, _ in groups for t in ap.apar_group_unfinished(grp)]
            max_live = max(max_live, len(live))
            q = quantise(0.6 * rng.standard_normal((len(live), n_q, d)).astype(np.float32), dtype)
            qd = to_dev(q, dtype)
            out = torch.empty_like(qd)
            ap.apar_decode_attention(pool.handle, qd, live, out)
            torch.cuda.synchronize()
            err = float(np.abs(to_host(out) - dense.decode(q, live)).max())
            worst = max(worst, err)
            assert err <= 2e-2, f"step {steps}: {err}"
            for grp, o, tid, ts in groups:
                todo = o.unfinished()
                if not todo:
                    continue
                xs = ts.sample([s.last_token for s in todo], [len(s.tokens) for s in todo], len(o.G))
                forkers = [s for s in todo if s.last_token == FORK]
                before = len(o.G)
                appended = o.step(xs)
                k, v = rows(len(appended))
                info = ap.apar_group_step(grp, xs, to_dev(k, dtype), to_dev(v, dtype))
                assert info.n_rows_appended == len(appended)
                new_ids = [t for t in ap.apar_group_unfinished(grp) if t not in tid.values()]
                for s, c in zip(forkers, o.G[before:]):
                    (kid,) = dense.fork(tid[s.sid], 1)
                    tid[c.sid] = kid
                assert sorted(new_ids) == sorted(tid[c.sid] for c in o.G[before:] if not c.finished)
                for i, s in enumerate(appended):
                    dense.append(tid[s.sid], k[i:i + 1], v[i:i + 1])
                for s, x in zip(todo, xs):
                    if x == EOS:
                        dense.free(tid[s.sid])
            steps += 1
        for grp, o, _, _ in groups:
            assert ap.apar_group_restore(grp) == o.restore()
            gi = ap.apar_group_get_info(grp)
            assert gi.max_cached_tokens == o.max_cached and gi.attended_tokens == o.attended
            ap.apar_group_destroy(grp)
        st = ap.apar_pool_stats(pool.handle)
        assert st.live_threads == 0 and st.free_blocks == st.total_blocks
        assert max_live > 8, "the groups should have forked"
        print(f"controller loop: {steps} steps, up to {max_live} threads, worst max abs err {worst:.2e}")
