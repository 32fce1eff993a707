"""apar_decode_attention_fixed (the entry point that allocates nothing) against apar_decode_attention.

Same plan, same kernels, only the home of the plan tables and partial results differs (the library's
static device workspace instead of allocated staging memory), so the two outputs must agree bit for bit;
the oracle is compared as well, to the tolerance of the other parity tests.  Two calls in a row on one
stream, the second with a smaller input, then a call that exceeds the workspace."""
import numpy as np
import pytest

import paper_2401_06761_amd as ap
from apar_workloads import HeadConfig, make_config, manual_tree, step_q
from oracle import BlockLedger, DenseThreads

from harness import blocks_upper_bound, nested_wide_tree, pool_for, replay_trace, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def both_entries(w, pool, dense, live, step):
    import torch

    q = step_q(w, step, len(live))
    qd = to_dev(q, w.heads.dtype)
    # different fill patterns, so that a row neither call writes shows up
    ref = torch.full_like(qd, 7.0)
    got = torch.full_like(qd, -3.0)
    ap.apar_decode_attention(pool.handle, qd, live, ref)
    info_ref = ap.apar_last_plan_info(pool.handle)
    ap.apar_decode_attention_fixed(pool.handle, qd, live, got)
    info_fix = ap.apar_last_plan_info(pool.handle)
    torch.cuda.synchronize()
    assert info_ref.n_partial_rows == info_fix.n_partial_rows and info_ref.n_units == info_fix.n_units
    assert torch.equal(ref, got), f"fixed entry differs: max abs {float((ref.float() - got.float()).abs().max())}"
    want = dense.decode(q, live)
    err = float(np.abs(to_host(got) - want).max())
    assert err <= TOL[w.heads.dtype], f"max abs err {err}"
    return info_fix


@pytest.mark.parametrize("case", ["ht256_8", "wide_partials_bf16", "ragged_f32_chunked"])
def test_fixed_entry_matches_allocating_entry_twice_in_a_row(case):
    chunk = None
    if case == "ht256_8":
        w = make_config("ht256", n_requests=8, data_scale=1.0)
    elif case == "wide_partials_bf16":
        w = nested_wide_tree(HeadConfig(8, 2, 128, "bf16"), seed=5)  # sharing groups of more than 128 rows
        chunk = 4                                                     # and chunked segments: partial results
    else:
        w = manual_tree([-1, 0, 0, 0, 1, 1, 3, 3, 3, -1, -1, 10, 10], [1, 15, 16, 17, 1, 33, 16, 15, 2, 1, 47, 1, 130],
                        HeadConfig(4, 4, 64, "f32"), seed=11)
        chunk = 2
    N = blocks_upper_bound(w)
    hd = w.heads
    with pool_for(w, N) as pool:
        pool.kv.fill_(0xFF)
        if chunk:
            ap.apar_set_chunk_blocks(pool.handle, chunk)
        dense = DenseThreads(hd.n_q_heads, hd.n_kv_heads, hd.head_dim)
        live, _ = replay_trace(w, pool, BlockLedger(N), dense)
        info = both_entries(w, pool, dense, live, 0)
        if chunk:
            assert info.n_partial_rows > 0, "this case is meant to leave partial results in the workspace"
        # second call: a smaller input (every third thread), the workspace still holds the first call's tables
        fewer = live[::3]
        info2 = both_entries(w, pool, dense, fewer, 1)
        assert info2.n_threads == len(fewer) < info.n_threads
        # and the first input again
        both_entries(w, pool, dense, live, 2)


def test_fixed_entry_refuses_what_does_not_fit():
    import torch

    heads = HeadConfig(32, 32, 128, "bf16")
    # one thread of 420 blocks, one block per work unit: 420 partial rows x 32 heads x 130 floats > 6 MiB
    w = manual_tree([-1], [420 * 16], heads, seed=1, data_scale=0.5)
    N = blocks_upper_bound(w)
    with pool_for(w, N) as pool:
        dense = DenseThreads(32, 32, 128)
        live, _ = replay_trace(w, pool, BlockLedger(N), dense)
        ap.apar_set_chunk_blocks(pool.handle, 1)
        q = step_q(w, 0, 1)
        qd = to_dev(q, "bf16")
        out = torch.full_like(qd, 5.0)
        with pytest.raises(ap.AparError) as e:
            ap.apar_decode_attention_fixed(pool.handle, qd, live, out)
        assert e.value.status == -7 and "workspace" in str(e.value)
        torch.cuda.synchronize()
        assert bool((out == 5.0).all()), "a refused call must not touch the output"
        # the allocating entry takes the same call, and the fixed one takes it with fewer chunks
        ref = torch.empty_like(qd)
        ap.apar_decode_attention(pool.handle, qd, live, ref)
        ap.apar_set_chunk_blocks(pool.handle, 64)
        ap.apar_decode_attention_fixed(pool.handle, qd, live, out)
        torch.cuda.synchronize()
        want = dense.decode(q, live)
        assert float(np.abs(to_host(out) - want).max()) <= 2e-2
        assert float(np.abs(to_host(ref) - want).max()) <= 2e-2
