"""A synthetic caller of the C ABI: builds a fork-tree workload in a pool and runs decode steps.

It plays the part of the decoding controller (the loop of Alg. 1 that samples, forks, appends and
releases) with seeded synthetic rows in place of a model.  It holds no arithmetic of the method:
every step below is one call into libapar.  bench.py and the full-size parity test both drive
the library through it, so that what is timed is what is checked.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

from apar_workloads import Workload, build_trace, node_kv_device, rows_device

from . import binding as ap

TAG_Q, TAG_K, TAG_V = 1, 2, 3


@dataclass
class StepRecord:
    step: int
    bank: int
    live: List[int]                      # threads attended, in list order
    replaced: List[Tuple[int, int, int]]  # (list position, finished parent, child that took its place)


class TreeRun:
    """One workload resident in one pool."""

    def __init__(self, w: Workload, headroom_steps: int = 64, n_banks: int = 4, churn: float = 0.01,
                 device: str = "cuda:0", kv_of=node_kv_device):
        """kv_of(w, node index, device) -> (k, v) rows of a tree node's segment: the seeded recipe unless a
        caller brings rows of its own (a test whose values say which rows were read)."""
        import torch

        self.torch = torch
        self.w = w
        self.kv_of = kv_of
        self.device = device
        self.churn = churn
        hd = w.heads
        n_leaves = len(w.leaves())
        # every node's own blocks, one copied tail per node, and room for the rows the steps add
        base = sum((n.seg_len + 15) // 16 + 1 for n in w.nodes)
        grow = n_leaves * ((headroom_steps + 15) // 16 + 2)
        self.num_blocks = base + grow + 16
        self.pool = ap.Pool(hd.n_q_heads, hd.n_kv_heads, hd.head_dim, hd.dtype, self.num_blocks,
                            max_threads=len(w.nodes) + n_leaves * (headroom_steps + 2) + 16, device=device)
        self.h = self.pool.handle
        self.live: List[int] = []
        self.node_of: Dict[int, int] = {}      # thread id -> tree node it decodes for
        self.extra_rows: Dict[int, List[Tuple[int, int]]] = {}  # thread id -> (bank, row) appended by steps
        self.n_banks = n_banks
        self.banks = None
        self.out = None
        self.rng = np.random.Generator(np.random.PCG64([w.seed, 0xC4]))
        self.records: List[StepRecord] = []
        self.step_no = 0

    # -- construction ---------------------------------------------------------
    def build(self) -> None:
        w, h = self.w, self.h
        ops, live, live_nodes = build_trace(w)
        for op in ops:
            if op.kind == "create":
                assert ap.apar_thread_create(h) == op.tid
            elif op.kind == "append":
                k, v = self.kv_of(w, op.node, self.device)
                ap.apar_append_kv(h, op.tid, k, v, op.n_tokens)
            elif op.kind == "fork":
                assert tuple(ap.apar_fork(h, op.tid, len(op.children))) == op.children
            else:
                ap.apar_free_thread(h, op.tid)
        self.live = list(live)
        self.node_of = dict(zip(live, live_nodes))
        self.extra_rows = {t: [] for t in live}
        hd = w.heads
        n = len(self.live)
        self.banks = [(rows_device(w, TAG_Q, b, (n, hd.n_q_heads, hd.head_dim), self.device),
                       rows_device(w, TAG_K, b, (n, hd.n_kv_heads, hd.head_dim), self.device, kv=True),
                       rows_device(w, TAG_V, b, (n, hd.n_kv_heads, hd.head_dim), self.device, kv=True))
                      for b in range(self.n_banks)]
        self.out = self.torch.empty_like(self.banks[0][0])
        self.torch.cuda.synchronize()

    # -- one pass of the hot path ---------------------------------------------
    def step(self, record: bool = False) -> None:
        """(Pass record=True on every step of a run, or on none: the per-thread row log that the
        parity check reads is only kept up to date while recording.)
        fork + release (a few threads finish and a forked child carries on in their place),
        append one row per live thread, decode attention over all live threads."""
        h = self.h
        n = len(self.live)
        replaced = []
        n_churn = int(round(self.churn * n))
        if n_churn > 0:
            for pos in sorted(int(x) for x in self.rng.choice(n, size=n_churn, replace=False)):
                parent = self.live[pos]
                (child,) = ap.apar_fork(h, parent, 1)
                ap.apar_free_thread(h, parent)
                self.live[pos] = child
                if record:
                    self.node_of[child] = self.node_of.pop(parent)
                    self.extra_rows[child] = self.extra_rows.pop(parent)
                    replaced.append((pos, parent, child))
        bank = self.step_no % self.n_banks
        q, k, v = self.banks[bank]
        ids = np.asarray(self.live, dtype=np.int32)
        ap.apar_append_kv_batch(h, ids, k, v)
        ap.apar_decode_attention(h, q, ids, self.out)
        if record:
            for i, t in enumerate(self.live):
                self.extra_rows[t].append((bank, i))
            self.records.append(StepRecord(self.step_no, bank, list(self.live), replaced))
        self.step_no += 1

    def close(self) -> None:
        self.pool.close()


class SpecRun:
    """The speculative (multi-candidate) decode loop on one pool.

    Per step, in the order the step plan fixes: multi-candidate attention over all live threads,
    append of each thread's accepted candidate rows, release of the threads that finish, fork of the
    survivors that spawn a child (the child receives one row).  Sized from a dry run of the same
    plan on a bookkeeping-only pool, so the pool holds exactly the peak the trace needs (+ slack).
    """

    TAG_CQ, TAG_CK, TAG_CV, TAG_CHILD_K, TAG_CHILD_V = 11, 12, 13, 14, 15

    def __init__(self, w: Workload, n_steps: int, n_cand: int = 5, p_fork: float = 0.02, p_finish: float = 0.01,
                 device: str = "cuda:0", fixed_bank: bool = True, commit: bool = True):
        import torch

        from apar_workloads import SpecLoopPlan

        self.torch = torch
        self.w, self.n_steps, self.C, self.device = w, n_steps, n_cand, device
        self.p_fork, self.p_finish = p_fork, p_finish
        self.fixed_bank = fixed_bank
        self.commit = commit  # False: gather the accepted rows here and append them in a second pass
        self._Plan = SpecLoopPlan
        hd = w.heads
        # dry run: same ops, no device memory
        ops, live, live_nodes = build_trace(w)
        dry = ap.Pool(hd.n_q_heads, hd.n_kv_heads, hd.head_dim, hd.dtype, 1 << 22, max_threads=1 << 30, dry_run=True)
        for op in ops:
            if op.kind == "create":
                ap.apar_thread_create(dry.handle)
            elif op.kind == "append":
                ap.apar_append_kv(dry.handle, op.tid, None, None, op.n_tokens)
            elif op.kind == "fork":
                ap.apar_fork(dry.handle, op.tid, len(op.children))
            else:
                ap.apar_free_thread(dry.handle, op.tid)
        plan = SpecLoopPlan(list(live), len(w.nodes), w.seed, n_cand, p_fork, p_finish)
        peak_blocks = ap.apar_pool_stats(dry.handle).used_blocks
        peak_threads = len(live)
        for _ in range(n_steps):
            st = plan.next_step()
            ids = np.repeat(np.asarray(st.live, dtype=np.int32), st.accept_bits.sum(axis=1))
            ap.apar_append_kv_batch(dry.handle, ids, None, None)
            peak_blocks = max(peak_blocks, ap.apar_pool_stats(dry.handle).used_blocks)  # before the releases
            for t in st.finished:
                ap.apar_free_thread(dry.handle, t)
            for t in st.forked:
                ap.apar_fork(dry.handle, t, 1)
            if st.children:
                ap.apar_append_kv_batch(dry.handle, st.children, None, None)
            peak_blocks = max(peak_blocks, ap.apar_pool_stats(dry.handle).used_blocks)
            peak_threads = max(peak_threads, len(plan.live), len(st.live))
        self.threads_issued = ap.apar_pool_stats(dry.handle).threads_issued
        dry.close()
        self.peak_blocks, self.peak_threads = int(peak_blocks), int(peak_threads)
        self.pool = ap.Pool(hd.n_q_heads, hd.n_kv_heads, hd.head_dim, hd.dtype, self.peak_blocks + 64,
                            max_threads=self.threads_issued + 16, device=device)
        self.h = self.pool.handle
        self.live: List[int] = []
        self.plan = None
        self.step_no = 0
        self.bank = None
        self.out = None
        self._drawn = []  # step plans drawn ahead of time, next one last

    def build(self) -> None:
        w, h, hd = self.w, self.h, self.w.heads
        ops, live, _ = build_trace(w)
        for op in ops:
            if op.kind == "create":
                assert ap.apar_thread_create(h) == op.tid
            elif op.kind == "append":
                k, v = node_kv_device(w, op.node, self.device)
                ap.apar_append_kv(h, op.tid, k, v, op.n_tokens)
            elif op.kind == "fork":
                assert tuple(ap.apar_fork(h, op.tid, len(op.children))) == op.children
            else:
                ap.apar_free_thread(h, op.tid)
        self.live = list(live)
        self.plan = self._Plan(list(live), len(w.nodes), w.seed, self.C, self.p_fork, self.p_finish)
        n = self.peak_threads
        if self.fixed_bank:
            self.bank = self.candidates_for(-1, n)
            self.child_bank = self.child_rows_for(-1, n)
        self.out = self.torch.empty((n, self.C, hd.n_q_heads, hd.head_dim), dtype=self.pool.torch_dtype,
                                    device=self.device)
        self.torch.cuda.synchronize()

    # seeded inputs of one step (index -1: the bank shared by all steps of a timing run)
    def candidates_for(self, step: int, n: int):
        hd, C = self.w.heads, self.C
        return (rows_device(self.w, self.TAG_CQ, step + 1, (n, C, hd.n_q_heads, hd.head_dim), self.device),
                rows_device(self.w, self.TAG_CK, step + 1, (n, C, hd.n_kv_heads, hd.head_dim), self.device, kv=True),
                rows_device(self.w, self.TAG_CV, step + 1, (n, C, hd.n_kv_heads, hd.head_dim), self.device, kv=True))

    def child_rows_for(self, step: int, n: int):
        hd = self.w.heads
        return (rows_device(self.w, self.TAG_CHILD_K, step + 1, (n, hd.n_kv_heads, hd.head_dim), self.device, kv=True),
                rows_device(self.w, self.TAG_CHILD_V, step + 1, (n, hd.n_kv_heads, hd.head_dim), self.device, kv=True))

    def draw_ahead(self, n_steps: int) -> None:
        """Draws the step plans of the next n_steps iterations now (the plan depends on nothing the library
        returns), so that a timed loop does not pay for generating its own synthetic input."""
        ahead = [self.plan.next_step() for _ in range(n_steps)]
        self._drawn = ahead[::-1] + self._drawn

    def step(self):
        """One loop iteration; returns (step plan, q, cand_k, cand_v, out view, child k, child v)."""
        torch, h, C = self.torch, self.h, self.C
        st = self._drawn.pop() if self._drawn else self.plan.next_step()
        n = len(st.live)
        if self.fixed_bank:
            q, ck, cv = (x[:n] for x in self.bank)
        else:
            q, ck, cv = self.candidates_for(st.step, n)
        ids = np.asarray(st.live, dtype=np.int32)
        masks = torch.from_numpy(st.masks).to(self.device, non_blocking=True)
        out = self.out[:n]
        ap.apar_decode_attention_spec(h, q, ck, cv, masks, C, ids, out)
        # accepted rows, thread by thread, each chain root -> accepted node
        if self.commit:
            ap.apar_commit_candidates(h, ids, ck, cv, C, st.accept_masks)
        else:
            counts = st.accept_bits.sum(axis=1)
            rep_ids = np.repeat(ids, counts)
            flat = np.flatnonzero(st.accept_bits.reshape(-1)).astype(np.int64)  # i * C + c, thread-major
            idx = torch.from_numpy(flat).to(self.device, non_blocking=True)
            hd = self.w.heads
            k_acc = ck.reshape(n * C, hd.n_kv_heads, hd.head_dim).index_select(0, idx)
            v_acc = cv.reshape(n * C, hd.n_kv_heads, hd.head_dim).index_select(0, idx)
            ap.apar_append_kv_batch(h, rep_ids, k_acc, v_acc)
        for t in st.finished:
            ap.apar_free_thread(h, t)
        kk = vv = None
        if st.forked:
            for t, child in zip(st.forked, st.children):
                assert ap.apar_fork(h, t, 1) == [child]
            m = len(st.children)
            if self.fixed_bank:
                kk, vv = (x[:m] for x in self.child_bank)
            else:
                kk, vv = self.child_rows_for(st.step, m)
            ap.apar_append_kv_batch(h, np.asarray(st.children, dtype=np.int32), kk, vv)
        self.live = list(st.live_after)
        self.step_no += 1
        return st, q, ck, cv, out, kk, vv

    def close(self) -> None:
        self.pool.close()
