"""A seeded stand-in for the model's sampler: which token each unfinished sequence emits per step.

Ordinary tokens are drawn from [0, vocab); with probability p_fork a sequence emits [Fork] (while the
group is below its thread budget), with probability p_eos it emits [EOS].  A sequence never emits
[Fork] twice in a row, emits no [EOS] before min_len tokens and is forced to [EOS] at max_len tokens.  Draw order: per step, one uniform
and one token per unfinished sequence, in the order given.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

FORK, CHILD, EOS = -1, -2, -3


class TokenStream:
    def __init__(self, seed: int, vocab: int = 32000, p_fork: float = 0.04, p_eos: float = 0.01,
                 max_threads: int = 12, max_len: int = 400, min_len: int = 0):
        self.rng = np.random.Generator(np.random.PCG64([seed, 0x70C]))
        self.vocab, self.p_fork, self.p_eos = vocab, p_fork, p_eos
        self.max_threads, self.max_len, self.min_len = max_threads, max_len, min_len

    def sample(self, last_tokens: Sequence[int], lengths: Sequence[int], n_threads_so_far: int) -> List[int]:
        out = []
        budget = self.max_threads - n_threads_so_far
        for last, length in zip(last_tokens, lengths):
            u = self.rng.random()
            tok = int(self.rng.integers(0, self.vocab))
            if length + 1 >= self.max_len:
                tok = EOS
            elif u < self.p_fork and last != FORK and budget > 0:
                tok = FORK
                budget -= 1
            elif u < self.p_fork + self.p_eos and length >= self.min_len:
                tok = EOS
            out.append(tok)
        return out
