"""Test helper: the engine's driver interface on top of the ORACLE's token table, so that the host state
machine can be exercised and checked without a GPU.  (Only oracle/ is used here, never the GPU library.)"""
import numpy as np

from oracle import TokenTable


class OracleDriver:
    def __init__(self, block_tables, block_size=16):
        self.tt = TokenTable(block_tables, block_size)
        self.calls = []

    def serial(self, new_len, hint):
        self.calls.append(("serial", new_len.tolist()))
        return self.tt.append_serial(new_len)

    def mixed(self, new_len_branch, new_len_main, hint):
        self.calls.append(("mixed", new_len_branch.tolist(), new_len_main.tolist()))
        return self.tt.append_mixed(new_len_branch, new_len_main)

    def renumber(self, num_branches):
        self.calls.append(("renumber", np.asarray(num_branches).tolist()))
        self.tt.open_parallel(num_branches)

    def merge(self, which):
        self.calls.append(("merge", np.asarray(which).tolist()))
        self.tt.merge(which)


class ScriptedModel:
    """Stands in for the model: per sequence a main-branch script (the tokens it will "choose", in order) and,
    per parallel stage, one script per branch.  Given a step it returns the token that follows every row
    that wants one."""

    def __init__(self, main_scripts, stage_scripts):
        self.main = [list(m) for m in main_scripts]
        self.stages = [[[list(b) for b in st] for st in seq] for seq in stage_scripts]   # [seq][stage][branch]
        self.stage_no = [-1] * len(main_scripts)

    def __call__(self, engine, plan):
        out = []
        for r in range(plan.NQ):
            if not plan.wants_output[r]:
                continue
            s, k = int(plan.seq[r]), int(plan.branch[r])
            if k < 0:
                out.append(self.main[s].pop(0))
            else:
                out.append(self.stages[s][engine.seqs[s].stages - 1][k].pop(0))
        return out
