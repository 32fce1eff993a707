"""What a pool that keeps full KV blocks in fp8 holds (test infrastructure; plain numpy + torch's cast).

The paper itself caches bf16/fp16; halving the bytes per cached token is this build's extension of its
throughput-against-cache-memory setting (Sec. 3.3), so the definition is the library header's, written
out plainly: when the sixteenth slot of a block is written, the block's K values of one kv head (16 x d)
and its V values are each rounded to OCP e4m3 (4 exponent bits, 3 mantissa bits, largest magnitude 448, no
infinities), round to nearest even, after division by a scale s = the smallest power of two with
max|x| / s <= 448 (s = 1 for a tile of zeros); the block then holds code * s.  Attention over such a pool is
dense.attend over these values: nothing else in the oracle changes.

The rounding itself is torch's float8_e4m3fn cast (a library primitive as a step); tests/test_oracle_numeric.py
pins it to the format's definition by brute force over all 256 codes and over the ties between them.
"""
from __future__ import annotations

import numpy as np

FP8_MAX = 448.0


def tile_scale(x: np.ndarray) -> float:
    """Smallest power of two s with max|x| / s <= 448 (1.0 for all zeros)."""
    amax = float(np.abs(x).max()) if x.size else 0.0
    if not amax > 0.0:
        return 1.0
    e = int(np.ceil(np.log2(amax / FP8_MAX)))
    while amax / 2.0 ** e > FP8_MAX:   # guard the rounding of log2
        e += 1
    while amax / 2.0 ** (e - 1) <= FP8_MAX:
        e -= 1
    return 2.0 ** max(e, -126)


def round_e4m3(y: np.ndarray) -> np.ndarray:
    """fp64 array -> nearest e4m3 value (ties to even), saturating at +-448, as fp64."""
    import torch

    t = torch.from_numpy(np.clip(np.asarray(y, dtype=np.float64), -FP8_MAX, FP8_MAX).astype(np.float32))
    return t.to(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)


def sealed_tile(x: np.ndarray) -> np.ndarray:
    """The values a full block keeps of x = its K (or V) values of one kv head, any shape."""
    s = tile_scale(x)
    return round_e4m3(np.asarray(x, dtype=np.float64) / s) * s


def cached_rows(K: np.ndarray, V: np.ndarray):
    """K, V: [T, Hkv, d] rows of one thread as appended.  Returns what the pool holds of them: every complete
    run of sixteen rows rounded per (kv head) tile, the rows of the last, still filling block untouched."""
    K = np.array(K, dtype=np.float64)
    V = np.array(V, dtype=np.float64)
    T = K.shape[0]
    for b in range(T // 16):
        for h in range(K.shape[1]):
            K[16 * b:16 * b + 16, h] = sealed_tile(K[16 * b:16 * b + 16, h])
            V[16 * b:16 * b + 16, h] = sealed_tile(V[16 * b:16 * b + 16, h])
    return K, V
