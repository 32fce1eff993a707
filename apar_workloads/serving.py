"""Synthetic serving workload: requests and a stateless stand-in for the model's sampler.

A request is (id, prompt length, seed).  The token a sequence emits depends only on
(request seed, index of the sequence in its group, length of the sequence): a 64-bit mix of the
three gives a uniform u and an ordinary token id, so any caller - the serving loop of the library,
the plain-Python oracle loop - draws the same tokens without sharing state, for any batch order:
  * length + 1 >= max_len                                    -> [EOS]
  * u < p_fork, last token not [Fork], group below max_threads at the start of the step -> [Fork]
  * p_fork <= u < p_fork + p_eos and length >= start + min_new -> [EOS]   (start: the length the
    sequence began with: the prompt for a root, its parent's tokens plus [Child] for a child)
  * otherwise an ordinary token in [0, vocab).
Only root sequences (index 0) and their descendants exist; a child starts at its parent's length + 1.
The sequential ("flat") stand-in of the same request never forks and ends after a given number of
generated tokens: what an ordinary auto-regressive model would do for a response of that length.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

FORK, CHILD, EOS = -1, -2, -3
_M = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(a: np.ndarray, b: np.ndarray, c: np.ndarray) -> np.ndarray:
    """splitmix64-style finaliser over three integer arrays -> uint64."""
    with np.errstate(over="ignore"):
        x = (a.astype(np.uint64) * np.uint64(0x9E3779B97F4A7C15)) ^ (b.astype(np.uint64) * np.uint64(0xBF58476D1CE4E5B9)) \
            ^ (c.astype(np.uint64) * np.uint64(0x94D049BB133111EB))
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


@dataclass(frozen=True)
class SamplerConfig:
    vocab: int = 32000
    p_fork: float = 0.04
    p_eos: float = 0.012
    max_threads: int = 8
    min_new: int = 24      # no [EOS] before a sequence has generated this many tokens itself
    max_len: int = 600     # hard cap on a sequence's length (prompt included)


@dataclass(frozen=True)
class Request:
    rid: int
    prompt_len: int
    seed: int

    def prompt_tokens(self) -> List[int]:
        return [int(x) for x in (_mix(np.full(self.prompt_len, self.seed), np.arange(self.prompt_len),
                                      np.full(self.prompt_len, 7)) % np.uint64(32000))]


def make_requests(n: int, seed: int = 0, prompt_lo: int = 16, prompt_hi: int = 256) -> List[Request]:
    rng = np.random.Generator(np.random.PCG64([seed, 0x5E41]))
    lens = rng.integers(prompt_lo, prompt_hi + 1, size=n)
    return [Request(i, int(lens[i]), int(seed) * 1_000_003 + i) for i in range(n)]


def sample_tokens(cfg: SamplerConfig, req_seed, seq_index, length, last_token, start_len, group_size) -> np.ndarray:
    """One token per listed sequence.  All arguments are equal-length integer arrays (one entry per
    unfinished sequence): its request's seed, its index in its group, its length, its last token,
    the length it began with, and the number of sequences its group held when the step began."""
    req_seed = np.asarray(req_seed, dtype=np.int64)
    seq_index = np.asarray(seq_index, dtype=np.int64)
    length = np.asarray(length, dtype=np.int64)
    last_token = np.asarray(last_token, dtype=np.int64)
    h = _mix(req_seed, seq_index, length)
    u = (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    tok = ((h ^ (h >> np.uint64(17))) % np.uint64(cfg.vocab)).astype(np.int64)
    fork = (u < cfg.p_fork) & (last_token != FORK) & (np.asarray(group_size) < cfg.max_threads)
    eos = (u >= cfg.p_fork) & (u < cfg.p_fork + cfg.p_eos) & (length >= np.asarray(start_len) + cfg.min_new)
    tok = np.where(fork, FORK, np.where(eos, EOS, tok))
    return np.where(length + 1 >= cfg.max_len, EOS, tok).astype(np.int32)


def sample_flat(cfg: SamplerConfig, req_seed, length, target_len) -> np.ndarray:
    """The sequential stand-in: ordinary tokens until the sequence reaches target_len - 1, then [EOS]."""
    req_seed = np.asarray(req_seed, dtype=np.int64)
    length = np.asarray(length, dtype=np.int64)
    h = _mix(req_seed, np.zeros_like(length), length)
    tok = ((h ^ (h >> np.uint64(17))) % np.uint64(cfg.vocab)).astype(np.int64)
    return np.where(length + 1 >= np.asarray(target_len), EOS, tok).astype(np.int32)
