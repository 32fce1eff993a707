"""Seeded Q/K/V values for a workload.

Values are standard normal times the workload's data_scale, rounded ONCE to the
pool dtype here; the HIP library and the oracle both consume these rounded
values (the oracle widens them exactly to fp64), so a parity tolerance covers
only arithmetic, never input rounding.

Each tree node and each decode step has its own counter-based stream
(Philox keyed by (seed, kind, index)), so any node's rows can be regenerated
alone, e.g. for a sampled parity check at a size whose full data would not fit
in host memory.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

_KIND_NODE = 1
_KIND_STEP_Q = 2
_KIND_SPEC = 3
_KIND_CHILD_ROW = 4


def _stream(seed: int, kind: int, index: int) -> np.random.Generator:
    key = (np.uint64(seed) << np.uint64(8)) | np.uint64(kind)
    return np.random.Generator(np.random.Philox(key=[int(key), int(index)]))


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# Pools of type "bf16_fp8kv" keep full blocks in fp8 (OCP e4m3: 1 sign, 4 exponent, 3 mantissa bits, largest
# magnitude 448) with a power-of-two scale per tile that the library derives from the tile's largest
# magnitude.  K and V rows for such pools are rounded HERE, once, to a grid the library's rounding leaves
# untouched whatever tile a row ends up in: e4m3 under the fixed scale 2^-6 (magnitudes up to 7, plenty for
# N(0,1) data and below).  A tile's own scale is never larger than that, and every value of this grid is
# representable under any smaller power-of-two scale that covers the tile's maximum, so the library stores
# these values exactly and the oracle, given the same values, sees what the kernels see.  Queries stay bf16.
FP8_GRID_EXP = -6
FP8_MAX = 448.0


def round_to_fp8_grid(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest (ties to even) multiple-of-quantum value of e4m3 under the scale 2^FP8_GRID_EXP, as fp32."""
    y = np.ascontiguousarray(x, dtype=np.float64) / 2.0 ** FP8_GRID_EXP
    y = np.clip(y, -FP8_MAX, FP8_MAX)
    mag = np.abs(y)
    expo = np.floor(np.log2(np.maximum(mag, 2.0 ** -6)))          # binade; below 2^-6 the format is subnormal
    quantum = 2.0 ** (expo - 3)
    r = np.rint(y / quantum) * quantum                              # rint rounds ties to even
    return (r * 2.0 ** FP8_GRID_EXP).astype(np.float32)


def quantise(x: np.ndarray, dtype: str, kv: bool = False) -> np.ndarray:
    """Round fp32 values to what a pool of the given type holds and return them as fp32 (exactly representable).
    kv: the values are K or V rows (only matters for "bf16_fp8kv", whose queries and outputs are plain bf16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16" or (dtype == "bf16_fp8kv" and not kv):
        return bf16_bits_to_f32(round_to_bf16_bits(x))
    if dtype == "bf16_fp8kv":
        return round_to_fp8_grid(x)
    raise ValueError(dtype)


def _normal(gen: np.random.Generator, shape, scale: float, dtype: str, kv: bool = False) -> np.ndarray:
    x = gen.standard_normal(size=shape, dtype=np.float32) * np.float32(scale)
    return quantise(x, dtype, kv)


def node_kv(w, node_idx: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V rows of one tree node: two fp32 arrays [seg_len, n_kv_heads, head_dim]."""
    h = w.heads
    n = w.nodes[node_idx].seg_len
    gen = _stream(w.seed, _KIND_NODE, node_idx)
    shape = (n, h.n_kv_heads, h.head_dim)
    k = _normal(gen, shape, w.data_scale, h.dtype, kv=True)
    v = _normal(gen, shape, w.data_scale, h.dtype, kv=True)
    return k, v


def step_q(w, step: int, n_rows: int) -> np.ndarray:
    """Queries of one decode step: fp32 [n_rows, n_q_heads, head_dim]."""
    h = w.heads
    gen = _stream(w.seed, _KIND_STEP_Q, step)
    return _normal(gen, (n_rows, h.n_q_heads, h.head_dim), w.data_scale, h.dtype)


def spec_step_qkv(w, step: int, n_rows: int, n_cand: int):
    """Candidate q, k, v of one speculative step: q [n, C, Hq, d]; k, v [n, C, Hkv, d]."""
    h = w.heads
    gen = _stream(w.seed, _KIND_SPEC, step)
    q = _normal(gen, (n_rows, n_cand, h.n_q_heads, h.head_dim), w.data_scale, h.dtype)
    k = _normal(gen, (n_rows, n_cand, h.n_kv_heads, h.head_dim), w.data_scale, h.dtype, kv=True)
    v = _normal(gen, (n_rows, n_cand, h.n_kv_heads, h.head_dim), w.data_scale, h.dtype, kv=True)
    return q, k, v


def child_rows(w, step: int, n_rows: int):
    """K, V of the single row a freshly forked child receives: [n, Hkv, d] each."""
    h = w.heads
    gen = _stream(w.seed, _KIND_CHILD_ROW, step)
    shape = (n_rows, h.n_kv_heads, h.head_dim)
    return _normal(gen, shape, w.data_scale, h.dtype, kv=True), _normal(gen, shape, w.data_scale, h.dtype, kv=True)


# ---------------------------------------------------------------------------
# Device-side twins for full-size runs, where drawing gigabytes on the host would
# dominate the run.  Same recipe (standard normal * data_scale, rounded once to the
# pool dtype) from torch's generator on the GPU; values differ from the numpy
# streams above but are just as reproducible.  The oracle receives the very
# tensors that were handed to the library, copied to the host.
# ---------------------------------------------------------------------------
def _torch_normal(shape, scale: float, dtype: str, seed: int, device, kv: bool = False):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * float(scale)
    if dtype == "f32":
        return x
    if dtype == "bf16_fp8kv" and kv:  # the fixed fp8 grid of round_to_fp8_grid (torch's cast rounds to nearest even too)
        s = 2.0 ** FP8_GRID_EXP
        x = (x / s).clamp(-FP8_MAX, FP8_MAX).to(torch.float8_e4m3fn).to(torch.float32) * s
    return x.to(torch.bfloat16)


def node_kv_device(w, node_idx: int, device="cuda:0"):
    h = w.heads
    shape = (w.nodes[node_idx].seg_len, h.n_kv_heads, h.head_dim)
    base = (int(w.seed) << 40) + (int(node_idx) << 2)
    return (_torch_normal(shape, w.data_scale, h.dtype, base + 1, device, kv=True),
            _torch_normal(shape, w.data_scale, h.dtype, base + 2, device, kv=True))


def rows_device(w, tag: int, index: int, shape, device="cuda:0", kv: bool = False):
    """Any other seeded tensor of a run (queries, per-step rows): stream (tag, index).  kv: rows that will be cached."""
    h = w.heads
    seed = (int(w.seed) << 40) + (int(tag) << 32) + (int(index) << 2) + 3
    return _torch_normal(tuple(shape), w.data_scale, h.dtype, seed, device, kv)
