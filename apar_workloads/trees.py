"""Fork-tree shapes and their op traces.

A workload is a forest: one tree per request.  A node is one generation thread's
own segment (the tokens it generates itself); its ancestors' segments are the
prefix it shares.  Internal nodes stop after forking (they are freed right after
the fork), so the live threads of a finished trace are exactly the leaves.

Draw order (fixed; one numpy Generator(PCG64(seed)) stream per workload):
per request: prompt length, root segment, child count, then per child in order:
segment, fork coin, grandchild count, grandchild segments.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class HeadConfig:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str  # "f32", "bf16" or "bf16_fp8kv" (bf16 at the interface, full blocks cached in fp8)
    block_size: int = 16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes


@dataclass
class Node:
    idx: int
    request: int
    parent: int  # node index, -1 for a root
    seg_len: int  # tokens this thread appends itself (roots: prompt + own segment)
    children: List[int] = field(default_factory=list)
    depth: int = 0


@dataclass
class Workload:
    name: str
    heads: HeadConfig
    nodes: List[Node]
    n_requests: int
    seed: int
    data_scale: float  # Q, K, V are N(0,1) * data_scale before rounding to dtype

    def leaves(self) -> List[int]:
        return [n.idx for n in self.nodes if not n.children]

    def root_path(self, idx: int) -> List[int]:
        path = []
        while idx >= 0:
            path.append(idx)
            idx = self.nodes[idx].parent
        return path[::-1]

    def path_len(self, idx: int) -> int:
        return sum(self.nodes[i].seg_len for i in self.root_path(idx))

    def total_unique_tokens(self) -> int:
        return sum(n.seg_len for n in self.nodes)

    def total_leaf_path_tokens(self) -> int:
        return sum(self.path_len(i) for i in self.leaves())


@dataclass(frozen=True)
class TraceOp:
    """One call of the library's problem statement.

    kind: "create" (tid = new id), "append" (tid, node, n_tokens), "fork"
    (tid = parent, children = new ids), "free" (tid).
    Thread ids are the ones a monotone counter from 0 issues, in op order.
    """

    kind: str
    tid: int
    node: int = -1
    n_tokens: int = 0
    children: Tuple[int, ...] = ()


CONFIG_NAMES = ("tiny", "mha64", "ht256", "gqa1024", "spec128")

_MHA = dict(n_q_heads=32, n_kv_heads=32, head_dim=128, dtype="bf16")
_GQA = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16")


def _add(nodes: List[Node], request: int, parent: int, seg_len: int) -> int:
    idx = len(nodes)
    depth = 0 if parent < 0 else nodes[parent].depth + 1
    nodes.append(Node(idx=idx, request=request, parent=parent, seg_len=int(seg_len), depth=depth))
    if parent >= 0:
        nodes[parent].children.append(idx)
    return idx


def _lognormal_seg(rng: np.random.Generator) -> int:
    x = rng.lognormal(mean=4.5, sigma=0.6)
    return int(np.rint(min(max(x, 8.0), 512.0)))


def _depth2_forest(rng, n_requests: int, prompt_lo: int, prompt_hi: int) -> List[Node]:
    nodes: List[Node] = []
    for r in range(n_requests):
        prompt = int(rng.integers(prompt_lo, prompt_hi + 1))
        root = _add(nodes, r, -1, prompt + _lognormal_seg(rng))
        n_children = int(rng.integers(2, 11))
        for _ in range(n_children):
            child = _add(nodes, r, root, _lognormal_seg(rng))
            if rng.random() < 0.5:
                n_grand = int(rng.integers(2, 7))
                for _ in range(n_grand):
                    _add(nodes, r, child, _lognormal_seg(rng))
    return nodes


def tiny_tree() -> Workload:
    """One request, fp32: a 16-token prompt, 8 root tokens, then 3 children of 8, 5, 12."""
    nodes: List[Node] = []
    root = _add(nodes, 0, -1, 16 + 8)
    for n in (8, 5, 12):
        _add(nodes, 0, root, n)
    heads = HeadConfig(n_q_heads=2, n_kv_heads=2, head_dim=64, dtype="f32")
    return Workload("tiny", heads, nodes, 1, seed=0, data_scale=1.0)


def manual_tree(parents: Sequence[int], seg_lens: Sequence[int], heads: HeadConfig,
                seed: int = 0, data_scale: float = 1.0, name: str = "manual") -> Workload:
    """A forest given explicitly: parents[i] < i (or -1), in creation order."""
    nodes: List[Node] = []
    req_of = {}
    n_req = 0
    for i, (p, s) in enumerate(zip(parents, seg_lens)):
        if p < 0:
            req_of[i] = n_req
            n_req += 1
        else:
            if p >= i:
                raise ValueError("parents must precede children")
            req_of[i] = req_of[p]
        _add(nodes, req_of[i], p, s)
    return Workload(name, heads, nodes, n_req, seed=seed, data_scale=data_scale)


def make_config(name: str, seed: int = 0, n_requests: Optional[int] = None,
                data_scale: Optional[float] = None, kv_fp8: bool = False) -> Workload:
    """The five named configurations.  `n_requests` takes the first n requests of
    the same stream (a prefix of the full forest), for subsampled parity runs."""
    if name == "tiny":
        return tiny_tree()
    rng = np.random.Generator(np.random.PCG64(seed))
    scale = 1.0 / np.sqrt(128.0) if data_scale is None else float(data_scale)
    if kv_fp8:  # the same shapes on a pool that keeps full blocks in fp8
        w = make_config(name, seed, n_requests, data_scale)
        w.heads = HeadConfig(w.heads.n_q_heads, w.heads.n_kv_heads, w.heads.head_dim, "bf16_fp8kv")
        w.name = name + "_fp8kv"
        return w
    if name == "mha64":
        n_req = 64 if n_requests is None else n_requests
        nodes: List[Node] = []
        for r in range(n_req):
            prompt = int(rng.integers(256, 1025))
            root = _add(nodes, r, -1, prompt + 64)
            k = int(rng.integers(4, 9))
            for _ in range(k):
                _add(nodes, r, root, int(rng.integers(64, 257)))
        return Workload(name, HeadConfig(**_MHA), nodes, n_req, seed, scale)
    if name == "ht256":
        n_req = 256 if n_requests is None else n_requests
        return Workload(name, HeadConfig(**_MHA), _depth2_forest(rng, n_req, 128, 512), n_req, seed, scale)
    if name == "gqa1024":
        n_req = 1024 if n_requests is None else n_requests
        return Workload(name, HeadConfig(**_GQA), _depth2_forest(rng, n_req, 1024, 4096), n_req, seed, scale)
    if name == "spec128":
        n_req = 128 if n_requests is None else n_requests
        return Workload(name, HeadConfig(**_MHA), _depth2_forest(rng, n_req, 128, 512), n_req, seed, scale)
    raise ValueError(f"unknown config {name!r}")


def build_trace(w: Workload) -> Tuple[List[TraceOp], List[int], List[int]]:
    """Request-major, depth-first op trace.

    Per node: (root only) create; append its segment; if it has children: fork
    them all at once, free the node, then recurse into each child in order.
    Returns (ops, live thread ids ascending, node index of each live thread).
    """
    ops: List[TraceOp] = []
    next_tid = 0
    tid_of = {}
    live: List[Tuple[int, int]] = []

    def visit(idx: int) -> None:
        nonlocal next_tid
        node = w.nodes[idx]
        tid = tid_of[idx]
        if node.seg_len > 0:
            ops.append(TraceOp("append", tid, node=idx, n_tokens=node.seg_len))
        if node.children:
            kids = tuple(range(next_tid, next_tid + len(node.children)))
            next_tid += len(kids)
            for c, k in zip(node.children, kids):
                tid_of[c] = k
            ops.append(TraceOp("fork", tid, children=kids))
            ops.append(TraceOp("free", tid))
            for c in node.children:
                visit(c)
        else:
            live.append((tid, idx))

    for node in w.nodes:
        if node.parent < 0:
            tid_of[node.idx] = next_tid
            ops.append(TraceOp("create", next_tid))
            next_tid += 1
            visit(node.idx)
    live.sort()
    return ops, [t for t, _ in live], [n for _, n in live]
