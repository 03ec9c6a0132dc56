"""The C writing of the oracle's attention (oracle/attention_ref.c: plain loops, OpenMP, no BLAS) behind
the interface of oracle.attention.attend.

TEST INFRASTRUCTURE (see oracle/__init__.py).  Two uses: the pins of tests/test_oracle_attention.py run
against it as well (two independent writings of Eq. 1 check each other), and bench.py's cpu_baseline
times it on the host's cores.  The mask still comes from TokenTable.dense_mask; rows are gathered with
numpy indexing; everything after that is the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

from .token_table import StepMeta, TokenTable

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "attention_ref.c")
LIB = os.path.join(_HERE, "libaspd_oracle.so")
_lib = None
last_threads = 1


def build(verbose: bool = False) -> str:
    cmd = [os.environ.get("CC", "gcc"), "-O2", "-fopenmp", "-shared", "-fPIC", "-o", LIB, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
            build()
        L = C.CDLL(LIB)
        L.aspd_oracle_attend.restype = C.c_int
        L.aspd_oracle_attend.argtypes = [C.c_void_p] * 4 + [C.c_int] * 5 + [C.c_double, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def attend_c(table: TokenTable, meta: StepMeta, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
             scale: float | None = None, rows=None, shared_mask: bool = False):
    """Same contract as oracle.attention.attend."""
    global last_threads
    NQ, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    qf = np.ascontiguousarray(q.to(torch.float64).numpy())
    out = np.full((NQ, Hq, D), np.nan)
    lse = np.full((NQ, Hq), np.nan)
    want = np.arange(NQ) if rows is None else np.asarray(rows, dtype=np.int64)
    for s in np.unique(meta.q_seq[want]):
        idx = want[meta.q_seq[want] == s]
        mask = np.ascontiguousarray(table.dense_mask(int(s), meta.logical_slot[idx], shared=shared_mask).astype(np.uint8))
        phys = table.physical_slots(int(s))
        blk = torch.from_numpy(phys // table.block_size)
        off = torch.from_numpy(phys % table.block_size)
        k_rows = np.ascontiguousarray(k_cache[blk, :, off].to(torch.float64).numpy())     # [T][Hkv][D]
        v_rows = np.ascontiguousarray(v_cache[blk, :, off].to(torch.float64).numpy())
        qs = np.ascontiguousarray(qf[idx])
        o = np.empty((idx.size, Hq, D))
        l = np.empty((idx.size, Hq))
        last_threads = lib().aspd_oracle_attend(qs.ctypes.data, k_rows.ctypes.data, v_rows.ctypes.data, mask.ctypes.data,
                                                int(idx.size), int(phys.size), int(Hq), int(Hkv), int(D), float(scale),
                                                o.ctypes.data, l.ctypes.data)
        out[idx] = o
        lse[idx] = l
    return out, lse
