"""The serving loop in plain Python (TEST INFRASTRUCTURE): a first-come-first-served queue of requests
over one block ledger, Algorithm 1 per request (controller.SequenceGroup), admission control and
preemption by recomputation.  The paper serves through an existing paged-attention engine and states
only the shape of the experiment (Sec. 3.3, App. C.2: all requests queued at the start, a cap on
concurrent requests, over-admission leads to swapping or recomputation); the policy written out here
is this build's reading, stated in the library header as well:

  admit    head of the queue only, while fewer than max_running requests run and
           free_blocks - ceil(prompt / 16) >= watermark;
  step     fork every sequence whose last token is [Fork], append all rows of all requests as one
           batch; if the ledger cannot hold them, undo the forks, release the most recently admitted
           running request (it returns to the head of the queue and restarts from its prompt) and try
           again without it; the oldest running request is never released - if the step does not fit
           with it alone the pool is too small for it and the step raises OutOfBlocks (no step applied,
           the requests released so far stay in the queue);
  after    sequences that drew [EOS] are released at once (early release, Sec. 2.4 feature 2);
           requests with no unfinished sequence leave with Restore(r) as their output.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

from .controller import EOS, FORK, SequenceGroup
from .ledger import BlockLedger, OutOfBlocks


class ServingOracle:
    def __init__(self, ledger: BlockLedger, max_running: int, watermark: int):
        self.led, self.max_running, self.watermark = ledger, max_running, watermark
        self.waiting: List[Tuple[int, int, List[int]]] = []  # (order, rid, prompt)
        self.running: List[dict] = []
        self.finished: List[Tuple[int, List[int], SequenceGroup]] = []
        self.order = 0
        self.steps = self.preemptions = self.admissions = self.generated = 0
        self.peak_used = self.peak_threads = 0

    def submit(self, rid: int, prompt: Sequence[int]) -> None:
        self.waiting.append((self.order, rid, list(prompt)))
        self.order += 1

    def admit(self) -> List[int]:
        """Returns the ids admitted, in order."""
        got = []
        while self.waiting and len(self.running) < self.max_running:
            order, rid, prompt = self.waiting[0]
            need = (len(prompt) + 15) // 16
            if self.led.free_blocks() - need < self.watermark:
                break
            t = self.led.create()
            self.led.append(t, len(prompt))
            g = SequenceGroup(prompt)
            self.running.append({"rid": rid, "order": order, "g": g, "tid": {0: t}, "prompt": prompt,
                                 "start": {0: len(prompt)}})
            self.waiting.pop(0)
            self.admissions += 1
            got.append(rid)
        self.peak_used = max(self.peak_used, self.led.used_blocks())
        return got

    def batch(self) -> List[dict]:
        out = []
        for r in self.running:
            g = r["g"]
            for s in g.unfinished():
                out.append({"request_id": r["rid"], "thread": r["tid"][s.sid], "seq_index": s.sid,
                            "last_token": s.last_token, "length": len(s.tokens), "start_len": r["start"][s.sid],
                            "group_size": len(g.G)})
        return out

    def _requeue(self, n_live: int) -> None:
        """The requests released in this step go back to the queue, in submission order."""
        for r in self.running[n_live:]:
            self.waiting.append((r["order"], r["rid"], r["prompt"]))
        self.waiting.sort(key=lambda w: w[0])
        self.running = self.running[:n_live]

    def step(self, sampled: Sequence[int]) -> dict:
        """Applies one step; returns what the library's step info reports plus, for a caller that mirrors
        the rows elsewhere: the (running index, row index) and the thread of every appended row, the
        (parent, child) thread pairs forked and the threads released, all in order."""
        ofs = [0]
        for r in self.running:
            ofs.append(ofs[-1] + len(r["g"].unfinished()))
        assert ofs[-1] == len(sampled)
        n_live = len(self.running)
        preempted = 0
        while True:
            kids_of: List[List[int]] = []
            rows: List[int] = []
            row_src: List[Tuple[int, int]] = []
            forks: List[Tuple[int, int]] = []
            for ri in range(n_live):
                r = self.running[ri]
                kids = []
                k = 0
                for s in r["g"].unfinished():
                    if s.last_token == FORK:
                        (c,) = self.led.fork(r["tid"][s.sid], 1)
                        forks.append((r["tid"][s.sid], c))
                        kids.append(c)
                        rows.append(c)
                        row_src.append((ri, k))
                        k += 1
                    rows.append(r["tid"][s.sid])
                    row_src.append((ri, k))
                    k += 1
                kids_of.append(kids)
            try:
                if rows:
                    self.led.append_batch(rows)
                break
            except OutOfBlocks:
                for kids in kids_of:
                    for c in kids:
                        self.led.free(c)
                if n_live <= 1:
                    self._requeue(n_live)
                    raise
                victim = self.running[n_live - 1]
                for s in victim["g"].unfinished():  # release in creation order
                    self.led.free(victim["tid"][s.sid])
                n_live -= 1
                preempted += 1
                self.preemptions += 1
        self._requeue(n_live)
        info = {"n_preempted": preempted, "n_forked": 0, "n_finished_sequences": 0, "n_finished_requests": 0,
                "n_rows_appended": len(rows), "rows": row_src, "row_threads": rows, "forks": forks, "freed": []}
        batch = 0
        for ri, r in enumerate(self.running):
            g = r["g"]
            todo = g.unfinished()
            xs = list(sampled[ofs[ri]:ofs[ri + 1]])
            before = len(g.G)
            g.step(xs)
            for c, t in zip(g.G[before:], kids_of[ri]):
                r["tid"][c.sid] = t
                r["start"][c.sid] = len(c.tokens)
            info["n_forked"] += len(g.G) - before
            for s, x in zip(todo, xs):
                if x == EOS:
                    self.led.free(r["tid"][s.sid])
                    info["freed"].append(r["tid"][s.sid])
                    info["n_finished_sequences"] += 1
            batch += len(xs)
        self.steps += 1
        self.generated += batch
        self.peak_threads = max(self.peak_threads, batch)
        self.peak_used = max(self.peak_used, self.led.used_blocks())
        keep = []
        for r in self.running:
            if r["g"].is_finished():
                self.finished.append((r["rid"], r["g"].restore(), r["g"]))
                info["n_finished_requests"] += 1
            else:
                keep.append(r)
        self.running = keep
        info["n_running"] = len(keep)
        return info
