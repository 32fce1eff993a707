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
                 device: str = "cuda:0"):
        import torch

        self.torch = torch
        self.w = w
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
                k, v = node_kv_device(w, op.node, self.device)
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
                       rows_device(w, TAG_K, b, (n, hd.n_kv_heads, hd.head_dim), self.device),
                       rows_device(w, TAG_V, b, (n, hd.n_kv_heads, hd.head_dim), self.device))
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
