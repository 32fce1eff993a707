"""CPU oracle for fork-tree paged-KV decode attention.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this; only tests, the smoke check and the
benchmark's cpu_baseline leg do.  It shares no code with the HIP library.

Two independent halves:
  * dense.py   - numeric: every thread owns a fully materialised fp64 copy of
                 its token rows (prefix deep-copied on fork), attention is the
                 plain softmax definition.  No blocks, tables or merges.
  * ledger.py  - bookkeeping: an integer-only replay of the allocator policy
                 (block tables, refcounts, free list, copy-on-write count).
  * controller.py - Algorithm 1 (fork on [Fork], paragraph nodes, Restore) in plain Python.
  * serving.py - the serving loop (queue, admission, preemption) over controller + ledger.
  * fp8.py     - what a pool that keeps full blocks in fp8 holds of the rows it was given.
  * accounting.py - the paper's max-cached-tokens / attended-tokens metrics and
                 the resident-vs-copied-prefix byte counts.
"""
from .dense import DenseThreads, attend, attend_spec  # noqa: F401
from .ledger import BlockLedger, OutOfBlocks, InvalidThread  # noqa: F401
from . import accounting  # noqa: F401
from . import fp8  # noqa: F401
from . import controller  # noqa: F401
from . import serving  # noqa: F401
