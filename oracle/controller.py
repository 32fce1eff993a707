"""Algorithm 1 of the APAR paper (decoding with paragraph nodes), plain Python.  TEST INFRASTRUCTURE.

Sequences are private token lists (a fork deep-copies the parent's list, as in dense.py);
paragraph nodes are objects with first_child / next_sibling pointers (Sec. 2.2 "Paragraph tree");
one call of step() is one decoding step of Alg. 1 over the unfinished sequences; restore() is the
algorithm's Restore: a node, then its first child's subtree, then its next sibling's.  The two savings metrics of Sec. 3.4 are
counted by brute force: attended tokens = length of the sequence a token was predicted from;
cached tokens = number of distinct token identities reachable from the unfinished sequences
(every token carries the identity (sequence that generated it, index), and a fork copies identities).

Readings fixed here (the algorithm listing leaves them open): a child created in a step starts
decoding in the next step; the prompt is not part of the restored output (the root node starts
where the prompt ends); the forced [Child] token lies before its node's start, so it is not restored either.
"""
from __future__ import annotations

from typing import List, Optional

FORK, CHILD, EOS = -1, -2, -3


class PNode:
    def __init__(self, seq: "Sequence_", start: int):
        self.seq, self.start, self.end = seq, start, None
        self.first_child: Optional["PNode"] = None
        self.next_sibling: Optional["PNode"] = None


class Sequence_:
    def __init__(self, sid: int, tokens: List[int], idents: List[tuple]):
        self.sid = sid
        self.tokens = list(tokens)
        self.idents = list(idents)
        self.finished = False
        self.current_node: Optional[PNode] = None

    @property
    def last_token(self) -> int:
        return self.tokens[-1]

    def append_token(self, x: int) -> None:
        self.idents.append((self.sid, len(self.tokens)))
        self.tokens.append(x)


class SequenceGroup:
    def __init__(self, prompt: List[int]):
        p = Sequence_(0, [], [])
        for x in prompt:
            p.append_token(x)
        self.root = PNode(p, len(p.tokens))
        p.current_node = self.root
        self.G: List[Sequence_] = [p]
        self.attended = 0
        self.generated = 0
        self.max_cached = self.cached_tokens()

    def unfinished(self) -> List[Sequence_]:
        return [s for s in self.G if not s.finished]

    def is_finished(self) -> bool:
        return not self.unfinished()

    def cached_tokens(self) -> int:
        held = set()
        for s in self.unfinished():
            held.update(s.idents)
        return len(held)

    def _branch_off(self, parent: Sequence_) -> Sequence_:
        """parent ends in [Fork]: a detail thread branches off.  The new sequence starts as a copy of the
        parent plus the forced [Child] token.  In the paragraph tree the parent's open paragraph is closed
        where it stands; the detail paragraph hangs below it (first child) and whatever the parent writes
        from here on comes after it on the same level (next sibling)."""
        detail_seq = Sequence_(len(self.G), parent.tokens, parent.idents)
        detail_seq.append_token(CHILD)
        self.G.append(detail_seq)
        closed = parent.current_node
        closed.end = len(parent.tokens)
        closed.first_child = PNode(detail_seq, len(detail_seq.tokens))
        closed.next_sibling = PNode(parent, len(parent.tokens))
        detail_seq.current_node, parent.current_node = closed.first_child, closed.next_sibling
        return detail_seq

    def step(self, sampled: List[int]) -> List[Sequence_]:
        """One decoding step of Alg. 1 over the unfinished sequences, sampled[i] being the token drawn for
        the i-th of them.  Returns the sequences whose KV rows were appended, one entry per row, in order
        (the [Child] row of a new thread, then the sampled token's row of its parent)."""
        todo = self.unfinished()
        assert len(todo) == len(sampled)
        rows: List[Sequence_] = []
        for seq, token in zip(todo, sampled):
            assert token != CHILD
            self.attended += len(seq.tokens)   # the token was predicted from the whole sequence
            self.generated += 1
            if seq.last_token == FORK:
                rows.append(self._branch_off(seq))
            seq.append_token(token)
            rows.append(seq)
            seq.finished = token == EOS        # a finished sequence no longer counts in cached_tokens()
        self.max_cached = max(self.max_cached, self.cached_tokens())
        return rows

    def restore(self) -> List[int]:
        out: List[int] = []

        def rec(node: Optional[PNode]) -> None:
            if node is None:
                return
            end = len(node.seq.tokens) if node.end is None else node.end
            out.extend(node.seq.tokens[node.start:end])
            rec(node.first_child)
            rec(node.next_sibling)

        import sys

        sys.setrecursionlimit(max(10000, sys.getrecursionlimit()))
        rec(self.root)
        return out
