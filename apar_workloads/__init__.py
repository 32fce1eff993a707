"""Seeded synthetic fork-tree workloads (inputs only).

This package serves both the HIP library's callers (tests, bench) and the CPU
oracle.  It holds none of the method's arithmetic: no block tables, no
refcounts, no attention.  It only draws tree shapes, segment lengths and
Q/K/V values, and turns a tree into the op trace
(create / append / fork / free) that either side replays.
"""
from .trees import (  # noqa: F401
    HeadConfig,
    Node,
    Workload,
    TraceOp,
    make_config,
    tiny_tree,
    manual_tree,
    build_trace,
    CONFIG_NAMES,
)
from .data import (  # noqa: F401
    round_to_bf16_bits,
    bf16_bits_to_f32,
    node_kv,
    step_q,
    quantise,
    spec_step_qkv,
    child_rows,
    node_kv_device,
    rows_device,
)
from .spec_loop import SpecLoopPlan, SpecStep, draw_candidate_tree, mask_rows_from_parents  # noqa: F401
from .token_stream import TokenStream  # noqa: F401
from .serving import Request, SamplerConfig, make_requests, sample_flat, sample_tokens  # noqa: F401
