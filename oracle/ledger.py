"""Bookkeeping half of the oracle (test infrastructure; integers only).

Replays create / fork / append / free and yields every live thread's block
table, every block's refcount and the free count.  The paper fixes only the
invariants - a fork shares every prefix block and copies at most one
(Sec. 2.3 "Decoding"), and a finished thread releases the KV cache that belongs
only to it (Alg. 1 ReleaseCache, Sec. 2.4 feature 2).  The physical ids follow
from the policy below, which is this build's reading, not the paper's:

  * refcount(b) = number of live threads whose table holds b;
  * thread ids come from a counter starting at 0 and are never reused; a fork
    returns n consecutive ids; the parent stays live until freed;
  * free blocks form a LIFO stack whose first pops are 0, 1, 2, ...;
  * fork allocates and copies nothing (copy-on-write is lazy);
  * append, token by token in order: at a block boundary pop a fresh block;
    otherwise, if the tail block is shared (refcount > 1), pop a new block
    first, copy the filled slots into it, drop one reference from the old tail
    and swap the table entry; then write the row.  A sole owner writes in place;
  * append is transactional: if the pool cannot supply every block the whole
    call needs, nothing changes;
  * a batch append (one row per listed thread) goes through the list in order;
  * free walks the table from the last block to the first and pushes each block
    whose refcount reaches zero.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple


class OutOfBlocks(RuntimeError):
    pass


class InvalidThread(KeyError):
    pass


class ThreadCapacity(RuntimeError):
    pass


class BlockLedger:
    def __init__(self, num_blocks: int, block_size: int = 16, max_threads: int = 1 << 30):
        self.N = int(num_blocks)
        self.B = int(block_size)
        self.max_threads = int(max_threads)
        self.ref = [0] * self.N
        self.free_stack = list(range(self.N - 1, -1, -1))  # pop() yields 0 first
        self.len: Dict[int, int] = {}
        self.table: Dict[int, List[int]] = {}
        self.next_tid = 0
        self.cow_copies = 0
        # every (block, slot) written by the last append call and every copy it made
        self.last_writes: List[Tuple[int, int]] = []
        self.last_copies: List[Tuple[int, int, int]] = []  # (src, dst, filled slots)

    # -- helpers ---------------------------------------------------------
    def _need(self, t: int):
        if t not in self.len:
            raise InvalidThread(t)

    def _blocks_for(self, n_tokens: int) -> int:
        return (n_tokens + self.B - 1) // self.B

    def _pop(self) -> int:
        b = self.free_stack.pop()
        assert self.ref[b] == 0
        self.ref[b] = 1
        return b

    # -- the five operations --------------------------------------------
    def create(self) -> int:
        if self.next_tid >= self.max_threads:
            raise ThreadCapacity()
        t = self.next_tid
        self.next_tid += 1
        self.len[t] = 0
        self.table[t] = []
        return t

    def fork(self, parent: int, n_children: int) -> List[int]:
        self._need(parent)
        if n_children < 1:
            raise ValueError("n_children must be >= 1")
        if self.next_tid + n_children > self.max_threads:
            raise ThreadCapacity()
        kids = []
        for _ in range(n_children):
            t = self.next_tid
            self.next_tid += 1
            self.len[t] = self.len[parent]
            self.table[t] = list(self.table[parent])
            for b in self.table[t]:
                self.ref[b] += 1
            kids.append(t)
        return kids

    def _blocks_needed(self, t: int, n_tokens: int) -> int:
        L = self.len[t]
        need = self._blocks_for(L + n_tokens) - self._blocks_for(L)
        if n_tokens > 0 and L % self.B != 0 and self.ref[self.table[t][-1]] > 1:
            need += 1
        return need

    def _append_one(self, t: int) -> None:
        L = self.len[t]
        tab = self.table[t]
        if L % self.B == 0:
            tab.append(self._pop())
        else:
            tail = tab[-1]
            if self.ref[tail] > 1:
                new = self._pop()
                self.last_copies.append((tail, new, L % self.B))
                self.ref[tail] -= 1
                tab[-1] = new
                self.cow_copies += 1
        b = tab[-1]
        assert self.ref[b] == 1, "a shared block must never be written"
        self.last_writes.append((b, L % self.B))
        self.len[t] = L + 1

    def append(self, t: int, n_tokens: int) -> None:
        self._need(t)
        if n_tokens < 0:
            raise ValueError("n_tokens must be >= 0")
        if self._blocks_needed(t, n_tokens) > len(self.free_stack):
            raise OutOfBlocks()
        self.last_writes, self.last_copies = [], []
        for _ in range(n_tokens):
            self._append_one(t)

    def append_batch(self, threads: Sequence[int]) -> None:
        for t in threads:
            self._need(t)
        # blocks the whole call needs, following the in-order policy: a shared
        # tail stops being shared for later threads of the list once earlier
        # sharers have copied away from it
        sim_ref: Dict[int, int] = {}
        sim_len: Dict[int, int] = {}
        sim_tail_fresh: Dict[int, bool] = {}
        need = 0
        for t in threads:
            L = sim_len.get(t, self.len[t])
            if L % self.B == 0:
                need += 1
                sim_tail_fresh[t] = True
            elif not sim_tail_fresh.get(t, False):
                tail = self.table[t][-1]
                r = sim_ref.get(tail, self.ref[tail])
                if r > 1:
                    need += 1
                    sim_ref[tail] = r - 1
                    sim_tail_fresh[t] = True
            sim_len[t] = L + 1
        if need > len(self.free_stack):
            raise OutOfBlocks()
        self.last_writes, self.last_copies = [], []
        for t in threads:
            self._append_one(t)

    def commit_candidates(self, threads: Sequence[int], accept_masks: Sequence[int]) -> None:
        """Books of a multi-candidate commit: one appended row per accepted candidate, thread by thread in
        listed order (the same allocator walk as append_batch with each thread repeated)."""
        rows = []
        for t, m in zip(threads, accept_masks):
            rows += [t] * bin(int(m)).count("1")
        if rows:
            self.append_batch(rows)

    def free(self, t: int) -> None:
        self._need(t)
        for b in reversed(self.table[t]):
            self.ref[b] -= 1
            assert self.ref[b] >= 0
            if self.ref[b] == 0:
                self.free_stack.append(b)
        del self.len[t], self.table[t]

    # -- introspection ---------------------------------------------------
    def live(self) -> List[int]:
        return sorted(self.len)

    def used_blocks(self) -> int:
        return self.N - len(self.free_stack)

    def free_blocks(self) -> int:
        return len(self.free_stack)

    def vanilla_blocks(self) -> int:
        """Blocks a layout that copies every prefix on fork would hold for the live threads."""
        return sum(self._blocks_for(L) for L in self.len.values())

    def check_invariants(self) -> None:
        live_refs = [0] * self.N
        for t, tab in self.table.items():
            assert len(tab) == self._blocks_for(self.len[t]), "table length != ceil(len/B)"
            assert len(set(tab)) == len(tab), "a table must not repeat a block"
            for b in tab:
                live_refs[b] += 1
        assert live_refs == self.ref, "refcount != number of live tables holding the block"
        assert sum(self.ref) == sum(self._blocks_for(L) for L in self.len.values())
        used = sum(1 for r in self.ref if r > 0)
        assert used + len(self.free_stack) == self.N
        assert len(set(self.free_stack)) == len(self.free_stack)
        assert all(self.ref[b] == 0 for b in self.free_stack)
