"""Rotary position encoding of the new tokens of an append call, and their placement in the cache.

TEST INFRASTRUCTURE (see oracle/__init__.py).  Plain numpy, float64.

ASPD's position ids (Sec. 3.2, Eq. 4) reach the attention scores through the position encoding of
the model that is fine-tuned; both base models of Sec. 4 (Vicuna, Qwen2.5) use rotary encodings.
The paper does not restate that encoding, so it is taken from its definition (Su et al., RoFormer),
in the layout those model families use (a reading, listed in the design notes):

  * head_dim D is split into D/2 pairs (i, i + D/2), i = 0 .. D/2-1 ("rotate-half" layout);
  * pair i of a vector at position p is rotated by the angle p * theta**(-2i/D);
  * queries and keys are rotated, values are not.

The step that uses it: every new token's query row is rotated by its position id, its key row is
rotated and written to the cache at the token's physical slot, its value row is written as it is.
"""
from __future__ import annotations

import numpy as np


def rotate(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """x [n][H][D] float64, positions [n] -> rotated copy.  Definition written out: for every pair
    (a, b) = (x[i], x[i + D/2]):  a' = a cos(phi) - b sin(phi),  b' = b cos(phi) + a sin(phi)."""
    n, H, D = x.shape
    half = D // 2
    out = np.empty_like(x, dtype=np.float64)
    for i in range(half):
        freq = float(theta) ** (-2.0 * i / D)
        phi = positions.astype(np.float64) * freq              # [n]
        c, s = np.cos(phi)[:, None], np.sin(phi)[:, None]      # [n][1]
        a, b = x[:, :, i], x[:, :, i + half]
        out[:, :, i] = a * c - b * s
        out[:, :, i + half] = b * c + a * s
    return out


def rope_append(q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, position_ids: np.ndarray,
                slot_mapping: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, theta: float):
    """q [NQ][Hq][D], k_new / v_new [NQ][Hkv][D] (float64); caches [blocks][Hkv][block][D] are
    modified in place at slot_mapping (physical slot = block * block_size + offset).
    Returns the rotated q."""
    block_size = k_cache.shape[2]
    k_rot = rotate(k_new, position_ids, theta)
    for r in range(q.shape[0]):
        blk, off = divmod(int(slot_mapping[r]), block_size)
        k_cache[blk, :, off, :] = k_rot[r]
        v_cache[blk, :, off, :] = v_new[r]
    return rotate(q, position_ids, theta)
