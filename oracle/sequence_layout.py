"""Whole multi-stage sequences given by their layout, replayed through the token table.

TEST INFRASTRUCTURE (see oracle/__init__.py).  Plain Python.

Fig. 5 of the paper shows the two arrangements of a parallel stage's tokens; the training one lays the
branches one after the other ("sequentially due to teacher forcing").  A layout names, per sequence, its
runs in cache order: (0, n) = n main-branch tokens, (k, n) = the n tokens of the k-th branch of a parallel
stage, the branches of a stage numbered 1..K in order.  Nothing is computed here that the token table does
not already define: serial runs are serial appends (Eq. 4, first case), a stage is opened, filled by ONE
append of whole branches (which lays each branch contiguously) and merged (Sec. 3.3).
"""
from __future__ import annotations

import numpy as np

from .token_table import StepMeta, TokenTable


def stages_of(runs):
    """[(0, n) | (k, n)] -> [("main", n) | ("par", [n_1..n_K])]; raises on a numbering that is not 1..K."""
    out = []
    for b, n in runs:
        b, n = int(b), int(n)
        assert n >= 0 and b >= 0
        if b == 0:
            out.append(("main", n))
        elif b == 1:
            out.append(("par", [n]))
        else:
            assert out and out[-1][0] == "par" and len(out[-1][1]) == b - 1, "branches of a stage are numbered 1..K in order"
            out[-1][1].append(n)
    return out


def replay_layout(block_tables, block_size, layouts, pos_mode="same_seq"):
    """layouts[s]: the runs of sequence s.  Returns (table, meta): the token table after the last stage of
    every sequence has been merged, and the metadata of all its tokens as query rows."""
    tt = TokenTable(block_tables, block_size, pos_mode=pos_mode)
    assert len(layouts) == tt.B
    stages = [stages_of(r) for r in layouts]
    for t in range(max((len(st) for st in stages), default=0)):
        K = np.zeros(tt.B, dtype=np.int32)
        main = np.zeros(tt.B, dtype=np.int32)
        branch = []
        for s in range(tt.B):
            if t >= len(stages[s]):
                continue
            kind, what = stages[s][t]
            if kind == "main":
                main[s] = what
            else:
                K[s] = len(what)
                branch.extend(what)
        tt.open_parallel(K)
        tt.append_mixed(np.array(branch, dtype=np.int32), main)
        tt.merge()
    return tt, tt.all_tokens_meta()
