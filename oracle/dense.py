"""Numeric half of the oracle (test infrastructure; fp64; slow on purpose).

The method reaches exactly the plain result: a decoding token attends to every
token on its path to the root of the paragraph tree and to nothing else
(APAR paper, Sec. 2.2 "Training attention", Fig. 2 caption, Sec. 2.4 feature 3).
So the oracle is that definition written out.  Each thread keeps its own dense
copy of its rows; a fork deep-copies the parent's rows, which is the paper's own
contiguous layout without prefix sharing (App. C.1).

Readings fixed here (the paper is silent on them):
  * the query's own K,V row is attended (Sec. 2.2: a token sees itself under the causal mask):
    callers append the new token's row first, then decode over all len rows;
  * softmax scale is 1/sqrt(head_dim) unless given;
  * grouped-query attention: q head h reads kv head h // (Hq / Hkv);
  * multi-candidate step (Medusa-style verification, Sec. 3.2 / App. C.1):
    candidate c attends to all cached rows, then to candidate c' iff bit c' of
    mask row c is set; candidates' K,V are passed alongside and are not cached;
  * segment prefill / training mask: the queries of a segment are the thread's
    last m positions, whose rows are already cached; a query sees its own row.

Parity pins for every function here live in tests/test_oracle_numeric.py.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np


def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """out[h] = sum_j softmax_j(scale * <q[h], K[j, h//g]>) * V[j, h//g].

    q: [Hq, d]; K, V: [T, Hkv, d], T >= 1; all fp64.  Returns [Hq, d] fp64.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    n_q, d = q.shape
    T, n_kv, _ = K.shape
    if T < 1:
        raise ValueError("softmax over an empty set is undefined")
    g = n_q // n_kv
    out = np.empty((n_q, d), dtype=np.float64)
    for h in range(n_q):
        kv = h // g
        s = scale * (K[:, kv, :] @ q[h])
        s = s - s.max()
        p = np.exp(s)
        p = p / p.sum()
        out[h] = p @ V[:, kv, :]
    return out


def attend_spec(q: np.ndarray, K: np.ndarray, V: np.ndarray, cand_k: np.ndarray,
                cand_v: np.ndarray, mask_rows: np.ndarray, scale: float) -> np.ndarray:
    """Multi-candidate step for one thread.

    q: [C, Hq, d]; K, V: [T, Hkv, d] cached rows; cand_k, cand_v: [C, Hkv, d];
    mask_rows: [C] bit-rows.  Candidate c's key set = the T cached rows followed
    by the candidates c' whose bit is set in mask_rows[c].  Returns [C, Hq, d].
    """
    C = q.shape[0]
    out = np.empty(q.shape, dtype=np.float64)
    for c in range(C):
        sel = [cp for cp in range(C) if (int(mask_rows[c]) >> cp) & 1]
        Kc = np.concatenate([np.asarray(K, np.float64), np.asarray(cand_k, np.float64)[sel]], axis=0)
        Vc = np.concatenate([np.asarray(V, np.float64), np.asarray(cand_v, np.float64)[sel]], axis=0)
        out[c] = attend(q[c], Kc, Vc, scale)
    return out


class InvalidDenseThread(KeyError):
    pass


class DenseThreads:
    """Threads with privately materialised token rows."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, scale: Optional[float] = None):
        if n_q_heads % n_kv_heads:
            raise ValueError("n_q_heads must be a multiple of n_kv_heads")
        self.n_q, self.n_kv, self.d = n_q_heads, n_kv_heads, head_dim
        self.scale = float(scale) if scale else 1.0 / float(np.sqrt(head_dim))
        self._k: Dict[int, np.ndarray] = {}
        self._v: Dict[int, np.ndarray] = {}
        self._next = 0

    def _get(self, t: int):
        if t not in self._k:
            raise InvalidDenseThread(t)
        return self._k[t], self._v[t]

    def create(self) -> int:
        t = self._next
        self._next += 1
        self._k[t] = np.zeros((0, self.n_kv, self.d), dtype=np.float64)
        self._v[t] = np.zeros((0, self.n_kv, self.d), dtype=np.float64)
        return t

    def fork(self, parent: int, n_children: int) -> List[int]:
        k, v = self._get(parent)
        kids = []
        for _ in range(n_children):
            t = self._next
            self._next += 1
            self._k[t] = k.copy()
            self._v[t] = v.copy()
            kids.append(t)
        return kids

    def append(self, t: int, k: np.ndarray, v: np.ndarray) -> None:
        K, V = self._get(t)
        k = np.asarray(k, dtype=np.float64).reshape(-1, self.n_kv, self.d)
        v = np.asarray(v, dtype=np.float64).reshape(-1, self.n_kv, self.d)
        self._k[t] = np.concatenate([K, k], axis=0)
        self._v[t] = np.concatenate([V, v], axis=0)

    def commit_candidates(self, threads: Sequence[int], cand_k: np.ndarray, cand_v: np.ndarray,
                          accept_masks: Sequence[int]) -> None:
        """Commit of a multi-candidate step (Sec. 3.2 Medusa-APAR; App. C.1): thread threads[i] gains the
        candidates c with bit c of accept_masks[i] set, in ascending c, taken from cand_k[i, c], cand_v[i, c]
        ([n, C, Hkv, d]); the others are dropped."""
        for i, t in enumerate(threads):
            for c in range(cand_k.shape[1]):
                if (int(accept_masks[i]) >> c) & 1:
                    self.append(t, cand_k[i, c], cand_v[i, c])

    def free(self, t: int) -> None:
        self._get(t)
        del self._k[t], self._v[t]

    def length(self, t: int) -> int:
        return self._get(t)[0].shape[0]

    def rows(self, t: int):
        return self._get(t)

    def live(self) -> List[int]:
        return sorted(self._k)

    def logits(self, q: np.ndarray, t: int) -> np.ndarray:
        """scale * <q[h], K_t[j, h//g]> for every q head and cached row: [Hq, T]."""
        K, _ = self._get(t)
        g = self.n_q // self.n_kv
        q = np.asarray(q, dtype=np.float64)
        # row-wise products and sums, so a row's logit does not depend on how many rows follow it
        return np.stack([self.scale * (K[:, h // g, :] * q[h]).sum(axis=1) for h in range(self.n_q)])

    def decode(self, q: np.ndarray, threads: Sequence[int]) -> np.ndarray:
        """q: [n, Hq, d] -> [n, Hq, d]; row i attends over all rows of threads[i]."""
        q = np.asarray(q, dtype=np.float64)
        out = np.empty((len(threads), self.n_q, self.d), dtype=np.float64)
        for i, t in enumerate(threads):
            K, V = self._get(t)
            out[i] = attend(q[i], K, V, self.scale)
        return out

    def prefill(self, q: np.ndarray, threads: Sequence[int], m: Sequence[int]) -> np.ndarray:
        """Tree-masked attention for whole segments (Sec. 2.2 "Training attention": a token attends only to
        the tokens on its path to the root, causally; the same mask serves the prompt / segment prefill).

        The last m[i] rows of thread threads[i] are the query tokens' own rows: query r of thread i sits at
        position len_i - m[i] + r and attends to rows 0 .. that position of the thread (its ancestors' rows
        up to each fork point, then its own rows up to and including itself).
        q: [sum(m), Hq, d], thread 0's m[0] queries first.  Returns the same shape.
        """
        q = np.asarray(q, dtype=np.float64)
        out = np.empty(q.shape, dtype=np.float64)
        row = 0
        for t, mi in zip(threads, m):
            K, V = self._get(t)
            L = K.shape[0]
            if mi < 1 or mi > L:
                raise ValueError("m must be in 1..len")
            for r in range(mi):
                last = L - mi + r
                out[row] = attend(q[row], K[: last + 1], V[: last + 1], self.scale)
                row += 1
        return out

    def decode_spec(self, q: np.ndarray, cand_k: np.ndarray, cand_v: np.ndarray,
                    mask_rows: np.ndarray, threads: Sequence[int]) -> np.ndarray:
        """q: [n, C, Hq, d]; cand_k, cand_v: [n, C, Hkv, d]; mask_rows: [n, C] -> [n, C, Hq, d]."""
        q = np.asarray(q, dtype=np.float64)
        out = np.empty(q.shape, dtype=np.float64)
        for i, t in enumerate(threads):
            K, V = self._get(t)
            out[i] = attend_spec(q[i], K, V, cand_k[i], cand_v[i], mask_rows[i], self.scale)
        return out
