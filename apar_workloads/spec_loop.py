"""Step plans for the speculative (multi-candidate) decode loop.

Per step, over the live threads in ascending id order:
  1. every thread proposes C candidate tokens arranged as a random tree
     (parent[0] = -1, parent[c] ~ Uniform{0..c-1}, drawn per step as one vector
     over the threads for each c); candidate c may see the cached tokens plus
     itself and its ancestors among the candidates;
  2. one node a ~ Uniform{0..C-1} is accepted together with its ancestor chain;
     those rows are appended to the cache in root -> a order;
  3. each thread finishes with probability p_finish (it is freed);
  4. each survivor forks one child with probability p_fork (the parent
     continues); the child receives one extra row.
The plan only draws integers and coins; it keeps its own list of live ids
(ids are issued by a monotone counter, so it can predict the children's).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


def draw_candidate_tree(rng: np.random.Generator, n_cand: int) -> np.ndarray:
    parents = np.full(n_cand, -1, dtype=np.int64)
    for c in range(1, n_cand):
        parents[c] = int(rng.integers(0, c))
    return parents


def mask_rows_from_parents(parents: np.ndarray) -> np.ndarray:
    """Bit-rows of the candidate tree mask: bit c' of row c is set iff c' is c or an ancestor of c."""
    n = len(parents)
    rows = np.zeros(n, dtype=np.uint8)
    for c in range(n):
        bits = 0
        a = c
        while a >= 0:
            bits |= 1 << a
            a = int(parents[a])
        rows[c] = bits
    return rows


@dataclass
class SpecStep:
    step: int
    live: List[int]  # thread ids attended this step, ascending
    parents: np.ndarray  # [n, C] candidate-tree parents
    masks: np.ndarray  # [n, C] uint8 bit-rows
    accepted: List[List[int]]  # per thread: candidate indices root -> a
    finished: List[int]  # thread ids freed after the appends
    forked: List[int]  # surviving thread ids that fork one child
    children: List[int]  # the children's ids, same order as `forked`
    accept_bits: np.ndarray = None  # [n, C] bool: the same accepted sets as a matrix
    accept_masks: np.ndarray = None  # [n] uint8: the same again, bit c of byte i = candidate c of thread i


class SpecLoopPlan:
    def __init__(self, live: List[int], next_tid: int, seed: int, n_cand: int = 5,
                 p_fork: float = 0.02, p_finish: float = 0.01):
        self.live = sorted(live)
        self.next_tid = int(next_tid)
        self.n_cand = n_cand
        self.p_fork = p_fork
        self.p_finish = p_finish
        self.rng = np.random.Generator(np.random.PCG64([seed, 0x5BEC]))
        self.step = 0

    def next_step(self) -> SpecStep:
        """Draw order per step: for c = 1..C-1 one vector of parents over the live threads (ascending
        id), then the vector of accepted nodes, then the finish coins, then the survivors' fork coins."""
        rng, C = self.rng, self.n_cand
        live = list(self.live)
        n = len(live)
        parents = np.full((n, C), -1, dtype=np.int64)
        masks = np.zeros((n, C), dtype=np.uint8)
        masks[:, 0] = 1
        rows = np.arange(n)
        for c in range(1, C):
            parents[:, c] = rng.integers(0, c, size=n)
            masks[:, c] = (1 << c) | masks[rows, parents[:, c]]
        node = rng.integers(0, C, size=n)
        chain_bits = masks[rows, node]  # the accepted node with its ancestors; ancestors have smaller indices
        bits = np.unpackbits(chain_bits[:, None], axis=1, bitorder="little")[:, :C].astype(bool)
        accepted = [list(np.flatnonzero(b)) for b in bits] if n <= 4096 else _LazyChains(bits)
        fin = rng.random(n) < self.p_finish
        live_arr = np.asarray(live, dtype=np.int64)
        finished = live_arr[fin].tolist()
        survivors = live_arr[~fin]
        fk = rng.random(len(survivors)) < self.p_fork
        forked = survivors[fk].tolist()
        children = list(range(self.next_tid, self.next_tid + len(forked)))
        self.next_tid += len(forked)
        self.live = sorted(survivors.tolist() + children)
        st = SpecStep(self.step, live, parents, masks, accepted, finished, forked, children)
        st.accept_bits = bits
        st.accept_masks = chain_bits.astype(np.uint8)
        st.live_after = self.live  # the live set once this step's releases and forks are done
        self.step += 1
        return st


class _LazyChains:
    """accepted[i] computed on demand from the bit matrix (large steps never walk all of them in Python)."""

    def __init__(self, bits: np.ndarray):
        self.bits = bits

    def __len__(self):
        return self.bits.shape[0]

    def __getitem__(self, i):
        return list(np.flatnonzero(self.bits[i]))

    def __iter__(self):
        return (list(np.flatnonzero(b)) for b in self.bits)
