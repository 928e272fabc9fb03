"""CPU oracle for an 8-bit form of the precomputed chunk caches (arXiv 2511.17560 notes that KV-cache
quantisation is orthogonal to the method and names loading the caches as its limitation; the paper fixes no
format).

TEST INFRASTRUCTURE ONLY, like the other oracle files.

Format taken here (listed again in the design notes): per packed row and KV head, symmetric 8-bit codes with
one float32 scale,
    scale = max_c |x_c| / 127,      q_c = round_half_even(x_c / scale) clipped to [-127, 127],      x^_c = q_c * scale,
a row of zeros has scale 0 and codes 0.  Keys are quantised as they are cached (at chunk-local positions);
position recovery (Eq. 2) runs on the dequantised keys, and the realigned keys are rounded once to the storage
type, as in the unquantised path.  Values are dequantised and rounded once to the storage type.

Pinned by tests/test_oracle_q8.py.
"""
from __future__ import annotations

import numpy as np

from . import a3_oracle as ora


def quantize_q8(x):
    """x [T, H, d] -> (codes int8 [T, H, d], scale float32 [T, H])."""
    x = np.asarray(x, dtype=np.float64)
    amax = np.abs(x).max(axis=-1)
    scale = (amax / 127.0).astype(np.float32)
    safe = np.where(scale > 0, scale.astype(np.float64), 1.0)
    q = np.clip(np.rint(x / safe[..., None]), -127, 127)          # rint rounds halves to even
    q = np.where(scale[..., None] > 0, q, 0.0)
    return q.astype(np.int8), scale


def dequantize_q8(q, scale, dtype=np.float64):
    return np.asarray(q, dtype=dtype) * np.asarray(scale, dtype=dtype)[..., None]


def dequant_values(q, scale, storage, dtype=np.float64):
    """The value cache the path reads: dequantised, rounded once to the storage type."""
    return ora.store(dequantize_q8(q, scale, dtype), storage, dtype)


def rope_realign_q8(q, scale, chunk_start, chunk_len, chunk_delta, base, layout, storage, dtype=np.float64):
    """Eq. 2 on the dequantised keys; one rounding at the end, for every row (rows that are not turned --
    chunks at offset 0, question rows -- are not storage-exact here, unlike in the unquantised path)."""
    turned = ora.rope_realign(dequantize_q8(q, scale, dtype), chunk_start, chunk_len, chunk_delta, base, layout,
                              "exact", dtype)
    return ora.store(turned, storage, dtype)
