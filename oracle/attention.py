"""Eq. 1 of ASPD Sec. 3.2 in float64 with the explicit dense mask of Eq. 2-3.

TEST INFRASTRUCTURE (see oracle/__init__.py).  No tiling, no running softmax, no
split of the key range: per (sequence, query, head) the scores over ALL slots of
the sequence are formed, the mask is applied, and one softmax is taken.

Conventions the paper leaves open (listed in the design notes): grouped-query
heads map query head h to KV head h // (Hq // Hkv); scale 1/sqrt(head_dim) unless
given; natural exponent; lse = max + log(sum exp).
"""
from __future__ import annotations

import numpy as np
import torch

from .token_table import StepMeta, TokenTable


def _rows_f64(cache: torch.Tensor, phys_slots: np.ndarray, kv_head: int, block_size: int) -> np.ndarray:
    """[T][D] float64 rows of one KV head, read from the paged array [blocks][Hkv][block][D]."""
    blk = torch.from_numpy(phys_slots // block_size)
    off = torch.from_numpy(phys_slots % block_size)
    return cache[blk, kv_head, off].to(torch.float64).numpy()


def attend_queries(q_rows: np.ndarray, k_rows: np.ndarray, v_rows: np.ndarray, mask: np.ndarray,
                   scale: float):
    """softmax(q k^T * scale + M) v for query rows [n][D] against keys/values [T][D];
    mask bool [n][T] (True = visible, i.e. M = 0; False = M = -inf).  Returns (out [n][D], lse [n])."""
    scores = (q_rows @ k_rows.T) * scale
    scores = np.where(mask, scores, -np.inf)
    m = scores.max(axis=1, keepdims=True)
    p = np.exp(scores - m)
    denom = p.sum(axis=1, keepdims=True)
    out = (p @ v_rows) / denom
    lse = (m + np.log(denom))[:, 0]
    return out, lse


def attend(table: TokenTable, meta: StepMeta, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
           scale: float | None = None, rows=None, shared_mask: bool = False):
    """Attention for the tokens of one append call (any of: parallel decode step, branch chunk,
    serial step), each query attending what Eq. 2-3 let it see among ALL slots now in its sequence.

    q [NQ][Hq][D]; caches [blocks][Hkv][block][D].  `rows` restricts the work to some packed rows
    (for sampled checks at full size).  Returns float64 out [NQ][Hq][D] and lse [NQ][Hq]; rows not
    asked for hold NaN.
    """
    NQ, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    qf = q.to(torch.float64).numpy()
    out = np.full((NQ, Hq, D), np.nan)
    lse = np.full((NQ, Hq), np.nan)
    want = np.arange(NQ) if rows is None else np.asarray(rows, dtype=np.int64)
    for s in np.unique(meta.q_seq[want]):
        idx = want[meta.q_seq[want] == s]
        mask = table.dense_mask(int(s), meta.logical_slot[idx], shared=shared_mask)
        phys = table.physical_slots(int(s))
        for kvh in range(Hkv):
            k_rows = _rows_f64(k_cache, phys, kvh, table.block_size)
            v_rows = _rows_f64(v_cache, phys, kvh, table.block_size)
            for h in range(kvh * G, (kvh + 1) * G):
                o, l = attend_queries(qf[idx, h], k_rows, v_rows, mask, scale)
                out[idx, h] = o
                lse[idx, h] = l
    return out, lse
