"""Shared test plumbing: replay one op trace on the library, the ledger and the dense oracle."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

import paper_2401_06761_amd as ap
from apar_workloads import build_trace, node_kv
from oracle import BlockLedger, DenseThreads


def to_dev(x: np.ndarray, dtype: str, device="cuda:0"):
    """fp32 numpy values (already representable in `dtype`) -> GPU tensor of the pool dtype."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)
    return t if dtype == "f32" else t.to(torch.bfloat16)


def to_host(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def books_equal(handle, led: BlockLedger, check_blocks: Optional[Sequence[int]] = None) -> None:
    """Block tables, lengths, refcounts and counters of the library against the ledger, bit-exact."""
    for t in led.live():
        assert ap.apar_thread_len(handle, t) == led.len[t], f"len of thread {t}"
        assert ap.apar_thread_block_table(handle, t) == led.table[t], f"table of thread {t}"
    blocks = range(led.N) if check_blocks is None else check_blocks
    for b in blocks:
        assert ap.apar_block_refcount(handle, b) == led.ref[b], f"refcount of block {b}"
    st = ap.apar_pool_stats(handle)
    assert st.used_blocks == led.used_blocks() and st.free_blocks == led.free_blocks()
    assert st.live_threads == len(led.live()) and st.cow_copies == led.cow_copies
    assert st.threads_issued == led.next_tid
    assert st.bytes_resident == led.used_blocks() * st.block_bytes
    assert st.bytes_vanilla == led.vanilla_blocks() * st.block_bytes


def replay_trace(w, pool: "ap.Pool", led: Optional[BlockLedger] = None, dense: Optional[DenseThreads] = None,
                 dry_run: bool = False, dense_nodes: Optional[set] = None, check_each: bool = False):
    """Runs build_trace(w) on the library and, if given, on the ledger and the dense oracle.
    Returns (live thread ids ascending, their node indices)."""
    ops, live, live_nodes = build_trace(w)
    h = pool.handle
    for op in ops:
        if op.kind == "create":
            assert ap.apar_thread_create(h) == op.tid
            if led is not None:
                assert led.create() == op.tid
            if dense is not None:
                assert dense.create() == op.tid
        elif op.kind == "append":
            if dry_run:
                ap.apar_append_kv(h, op.tid, None, None, op.n_tokens)
            else:
                k, v = node_kv(w, op.node)
                ap.apar_append_kv(h, op.tid, to_dev(k, w.heads.dtype), to_dev(v, w.heads.dtype), op.n_tokens)
                if dense is not None:
                    dense.append(op.tid, k, v)
            if led is not None:
                led.append(op.tid, op.n_tokens)
        elif op.kind == "fork":
            assert tuple(ap.apar_fork(h, op.tid, len(op.children))) == op.children
            if led is not None:
                assert tuple(led.fork(op.tid, len(op.children))) == op.children
            if dense is not None:
                assert tuple(dense.fork(op.tid, len(op.children))) == op.children
        elif op.kind == "free":
            ap.apar_free_thread(h, op.tid)
            if led is not None:
                led.free(op.tid)
            if dense is not None:
                dense.free(op.tid)
        if check_each and led is not None:
            books_equal(h, led)
    return live, live_nodes


def pool_for(w, num_blocks: int, dry_run: bool = False, **kw) -> "ap.Pool":
    hd = w.heads
    return ap.Pool(hd.n_q_heads, hd.n_kv_heads, hd.head_dim, hd.dtype, num_blocks, dry_run=dry_run, **kw)


def blocks_upper_bound(w) -> int:
    """Enough blocks for any replay of w: every node's segment rounded up, plus one copy per node."""
    return sum((n.seg_len + 15) // 16 + 1 for n in w.nodes) + 4


def check_plan_covers_tables(handle, threads: Sequence[int], n_kv: int, rows_per_thread: int = 1) -> Dict[str, int]:
    """The exported plan must read, for every listed thread, exactly the blocks of its table, in
    order, through the partial-result rows on its path; and no block twice for one row group."""
    units = np.array(ap.apar_last_plan_export(handle, ap.APAR_PLAN_UNITS), dtype=np.int64).reshape(-1, 6)
    blocks = ap.apar_last_plan_export(handle, ap.APAR_PLAN_BLOCKS)
    sharers = ap.apar_last_plan_export(handle, ap.APAR_PLAN_SHARERS)
    path_ofs = ap.apar_last_plan_export(handle, ap.APAR_PLAN_PATH_OFS)
    path_ids = ap.apar_last_plan_export(handle, ap.APAR_PLAN_PATH_IDS)
    row_owner = {}
    for fam, (bo, nb, lv, so, ns, pb) in enumerate(units):
        assert nb >= 1 and 1 <= lv <= 16 and ns >= 1
        assert ns * rows_per_thread <= 64
        for j in range(ns):
            assert pb + j not in row_owner
            row_owner[pb + j] = (fam, sharers[so + j])
    assert len(path_ofs) == len(threads) + 1
    reads = 0
    for i, t in enumerate(threads):
        table = ap.apar_thread_block_table(handle, t)
        L = ap.apar_thread_len(handle, t)
        got: List[int] = []
        tokens = 0
        fams = []
        for p in path_ids[path_ofs[i]:path_ofs[i + 1]]:
            fam, who = row_owner[p]
            assert who == i
            bo, nb, lv = units[fam][:3]
            fams.append((bo, fam))
        for bo, fam in sorted(fams):  # block runs of one thread are laid out in table order
            _, nb, lv = units[fam][:3]
            got.extend(blocks[bo:bo + nb])
            tokens += (nb - 1) * 16 + lv
        assert got == table, f"thread {t}: plan reads {got}, table is {table}"
        assert tokens == L
    info = ap.apar_last_plan_info(handle)
    assert info.n_units == len(units) * n_kv and info.n_partial_rows == len(row_owner)
    uniq = set()
    for t in threads:
        uniq.update(ap.apar_thread_block_table(handle, t))
    assert info.unique_blocks == len(uniq) == len(blocks) == len(set(blocks))
    assert info.path_tokens == sum(ap.apar_thread_len(handle, t) for t in threads)
    for (bo, nb, lv, so, ns, pb) in units:
        reads += nb
    return {"unit_block_reads": reads, "unique_blocks": len(uniq)}
