"""Test helper: bring the ORACLE's token table to the state a workload describes.

Only oracle/ and the input generators are used here (never the GPU library)."""
import numpy as np

import aspd_workloads as W
from oracle import TokenTable


def table_with_prefix(wl) -> TokenTable:
    tt = TokenTable(wl.block_tables, wl.block_size)
    tt.append_serial(wl.prefix_len)
    return tt


def table_at(wl, branch_len) -> TokenTable:
    """Prefix, then a parallel stage whose branches hold branch_len[b] tokens, grown one token
    per active branch per step."""
    tt = table_with_prefix(wl)
    tt.open_parallel(wl.num_branches)
    for new_len in W.interleaved_history(branch_len):
        tt.append_parallel(new_len)
    return tt
