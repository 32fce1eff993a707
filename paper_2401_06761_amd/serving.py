"""A synthetic serving loop over the library's scheduler (apar_server_*): the caller's side of it.

Per step: admit from the queue, list the batch, run decode attention over the batch's threads, draw one
token per sequence from the stateless sampler that stands in for the model, apply the step.  Rows of
K, V and q come from fixed seeded banks (their values do not matter to the scheduler).  In "flat" mode
every request is decoded as one sequence of a given total length: what an ordinary auto-regressive
model would do for the same response (the paper's "Original" models).
"""
from __future__ import annotations

import time
from typing import Dict, List, Optional, Sequence

import numpy as np

from apar_workloads import Request, SamplerConfig, sample_flat, sample_tokens

from . import binding as ap


class ServingRun:
    def __init__(self, pool: "ap.Pool", requests: Sequence[Request], sampler: SamplerConfig, max_running: int,
                 watermark_blocks: int, flat_lengths: Optional[Dict[int, int]] = None, banks=None,
                 attention: bool = True):
        """banks: (q [B, Hq, d], k [R, Hkv, d], v [R, Hkv, d]) device tensors, or None on a dry-run pool.
        flat_lengths: request id -> total sequence length (prompt included) for the sequential stand-in."""
        self.pool, self.h = pool, pool.handle
        self.requests = {r.rid: r for r in requests}
        # seed of every request by id, for one vectorised look-up per step
        self._rids = np.array(sorted(self.requests), dtype=np.int64)
        self._seeds = np.array([self.requests[int(r)].seed for r in self._rids], dtype=np.int64)
        self._flat_target = None
        if flat_lengths is not None:
            self._flat_target = np.array([flat_lengths[int(r)] for r in self._rids], dtype=np.int64)
        self.sampler = sampler
        self.flat = flat_lengths
        self.banks = banks
        self.attention = attention and banks is not None
        self.srv = ap.apar_server_create(self.h, max_running, watermark_blocks)
        for r in requests:
            ap.apar_server_submit(self.srv, r.rid, r.prompt_tokens())
        self.outputs: Dict[int, List[int]] = {}
        self.infos: Dict[int, "ap.AparGroupInfo"] = {}
        self.trace: List[dict] = []
        self.keep_trace = False
        self.out = None

    def step(self) -> bool:
        """One scheduling + decode step.  False when nothing is left to do."""
        q, k, v = self.banks if self.banks is not None else (None, None, None)
        rows_cap = int(k.shape[0]) if k is not None else 1 << 40
        n_adm, _ = ap.apar_server_admit(self.srv, k, v, rows_cap)
        batch = ap.apar_server_batch(self.srv)
        n = len(batch)
        if n == 0:
            st = ap.apar_server_get_stats(self.srv)
            if st.n_waiting == 0:
                return False
            raise RuntimeError("the head of the queue does not fit an empty pool")
        if self.attention:
            if self.out is None or self.out.shape[0] < n:
                self.out = q.new_empty((max(n, q.shape[0]),) + tuple(q.shape[1:]))
            ap.apar_decode_attention(self.h, q[:n], batch["thread"], self.out[:n])
        seeds = self._seeds[np.searchsorted(self._rids, batch["request_id"])]
        if self.flat is None:
            sampled = sample_tokens(self.sampler, seeds, batch["seq_index"], batch["length"], batch["last_token"],
                                    batch["start_len"], batch["group_size"])
        else:
            target = self._flat_target[np.searchsorted(self._rids, batch["request_id"])]
            sampled = sample_flat(self.sampler, seeds, batch["length"], target)
        info = ap.apar_server_step(self.srv, sampled, k, v)
        if self.keep_trace:
            self.trace.append({"admitted": n_adm, "threads": batch["thread"].tolist(), "sampled": sampled.tolist(),
                               "n_preempted": info.n_preempted, "n_forked": info.n_forked,
                               "n_rows_appended": info.n_rows_appended,
                               "n_finished_requests": info.n_finished_requests})
        for _ in range(info.n_finished_requests):
            done = ap.apar_server_pop_finished(self.srv)
            if done is None:
                break
            rid, tokens, ginfo = done
            self.outputs[rid] = tokens
            self.infos[rid] = ginfo
        return True

    def run(self, max_steps: int = 1 << 30) -> dict:
        t0 = time.perf_counter()
        steps = 0
        while steps < max_steps and self.step():
            steps += 1
        while True:  # nothing should be left; a request the loop above did not collect shows up here
            done = ap.apar_server_pop_finished(self.srv)
            if done is None:
                break
            self.outputs[done[0]], self.infos[done[0]] = done[1], done[2]
        if self.banks is not None:
            import torch

            torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        st = ap.apar_server_get_stats(self.srv)
        return {"wall_s": wall, "steps": st.steps, "generated_tokens": st.generated_tokens,
                "useful_tokens": sum(len(t) for t in self.outputs.values()),
                "finished": st.n_finished, "admissions": st.n_admissions, "preemptions": st.n_preemptions,
                "peak_used_blocks": st.peak_used_blocks, "peak_running": st.peak_running,
                "peak_threads": st.peak_threads, "mean_batch": st.batch_sequences_total / max(st.steps, 1)}

    def close(self) -> None:
        if self.srv is not None:
            ap.apar_server_destroy(self.srv)
            self.srv = None
