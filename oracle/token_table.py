"""Token table of a serial-parallel decoded sequence, grown by replaying appends.

TEST INFRASTRUCTURE (see oracle/__init__.py).  Plain Python and numpy.

Follows ASPD Sec. 3.2 "Preliminaries" and Eq. 2-4.  A sequence is a succession of
stages; a serial stage has one main branch, a parallel stage has K parallel
branches.  Every token carries (stage, branch, index within its branch, position
id).  One KV cache per sequence is reused throughout (abstract, Sec. 2.3): a token's
logical slot is its index in the order the tokens were appended, and a merge moves
nothing.

Readings of the paper taken here (each is also listed in the design notes):
  * Position ids are 0-based: Eq. 4 minus one throughout (rotary encodings only see
    differences).
  * Eq. 4, main branch: position = number of tokens of all earlier timesteps, i.e.
    the count of tokens already in the sequence ("absolute positions in the
    flattened sequence").
  * Eq. 4, parallel branch: stage_start = position the first token of every branch
    takes = number of tokens before the stage; Delta = 0-based index of the token
    within its own branch ("shared position encodings at each timestamp").
  * Eq. 2 is read with self-visibility: visible iff S = 1 and (pos(i) > pos(j) or
    i = j); a strict test alone would leave the first token's row empty.
  * One append call lays its new tokens at the tail ordered by (branch index, token
    index).  A one-token-per-branch step therefore interleaves branches (the
    inference arrangement of Fig. 5) and a multi-token call lays each branch's chunk
    contiguously (the teacher-forcing arrangement of Fig. 5).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

MAIN = 0  # branch id of the main branch; parallel branches are 1..K within their stage


@dataclass
class StepMeta:
    """What one append call hands to the attention call that follows it."""

    cu_new: np.ndarray         # [NB+1] (parallel) or [B+1] (serial): first packed row of each branch / sequence
    cu_seq_new: np.ndarray     # [B+1]  first packed row of each sequence
    q_seq: np.ndarray          # [NQ]   sequence of each new token
    q_branch: np.ndarray       # [NQ]   global branch index (parallel) or -1 (serial)
    position_ids: np.ndarray   # [NQ]   Eq. 4, 0-based
    logical_slot: np.ndarray   # [NQ]   index of the token in its sequence's cache
    slot_mapping: np.ndarray   # [NQ]   int64 physical slot through the block table
    kv_len: np.ndarray         # [NQ]   number of keys the token attends to, itself included

    @property
    def NQ(self) -> int:
        return int(self.q_seq.shape[0])


class TokenTable:
    def __init__(self, block_tables: np.ndarray, block_size: int, pos_mode="same_seq"):
        """pos_mode: the position-id paradigm (Sec. 4.5.3).  "same_seq" is the one the paper adopts
        (Eq. 4: after a parallel stage the main branch continues at the number of tokens decoded so
        far).  The two it compares against, as read here: "same_max" - branches share positions in the
        same way, but the main branch continues right after the largest position any branch reached;
        ("fix", N) - branch k of a stage owns the pre-allocated interval [stage_start + k N,
        stage_start + (k+1) N) and the main branch continues after the last interval."""
        self.block_tables = np.asarray(block_tables)
        self.block_size = int(block_size)
        self.B = int(self.block_tables.shape[0])
        self.pos_mode = pos_mode
        self.fix_n = int(pos_mode[1]) if isinstance(pos_mode, tuple) else 0
        assert pos_mode in ("same_seq", "same_max") or (isinstance(pos_mode, tuple) and pos_mode[0] == "fix")
        self.next_main_pos = [0] * self.B        # position id the next main-branch token takes
        # per sequence, per logical slot
        self.stage = [[] for _ in range(self.B)]
        self.branch = [[] for _ in range(self.B)]
        self.index_in_branch = [[] for _ in range(self.B)]
        self.pos = [[] for _ in range(self.B)]
        # stage bookkeeping
        self.cur_stage = [0] * self.B            # stage number of the stage now being decoded
        self.cur_parallel = [False] * self.B
        self.stage_first_slot = [0] * self.B     # slot of the first token of the current stage
        self.stage_start_pos = [0] * self.B      # Eq. 4 stage_start of the current parallel stage
        self.tokens_in_branch = [[] for _ in range(self.B)]   # per branch of the current parallel stage
        self.main_count = [0] * self.B

    # ------------------------------------------------------------------ appends
    def _push(self, s: int, branch: int, t: int, pos: int) -> int:
        slot = len(self.pos[s])
        self.stage[s].append(self.cur_stage[s])
        self.branch[s].append(branch)
        self.index_in_branch[s].append(t)
        self.pos[s].append(pos)
        return slot

    def _push_main(self, s: int) -> int:
        """One main-branch token.  Same-Seq: its position is the number of tokens decoded before it, all
        branches included (Eq. 4, first case); the other paradigms continue from where the merge left
        the position counter."""
        pos = len(self.pos[s]) if self.pos_mode == "same_seq" else self.next_main_pos[s]
        slot = self._push(s, MAIN, self.main_count[s], pos)
        self.main_count[s] += 1
        self.next_main_pos[s] = pos + 1
        return slot

    def _branch_pos(self, s: int, k: int, t: int) -> int:
        """Token t (0-based) of branch k (0-based) of the running stage: Eq. 4, second case."""
        if self.fix_n:
            assert t < self.fix_n, "branch outgrew its pre-allocated interval"
            return self.stage_start_pos[s] + k * self.fix_n + t
        return self.stage_start_pos[s] + t

    def append_serial(self, new_len) -> StepMeta:
        """Main-branch tokens: new_len[s] of them for sequence s (Eq. 4 case 1)."""
        new_len = np.asarray(new_len)
        assert new_len.shape == (self.B,)
        rows = []
        for s in range(self.B):
            assert not self.cur_parallel[s], "merge before appending main tokens"
            for _ in range(int(new_len[s])):
                slot = self._push_main(s)
                rows.append((s, -1, slot))
        cu_new = np.zeros(self.B + 1, dtype=np.int32)
        np.cumsum(new_len, out=cu_new[1:])
        return self._step_meta(rows, cu_new)

    def open_parallel(self, num_branches) -> None:
        """Start a parallel stage with num_branches[s] branches (0 leaves the sequence serial).
        A sequence whose parallel stage is still running is named with the branch count it has and
        stays as it is: sequences switch stages independently of one another (Sec. 3.3)."""
        num_branches = np.asarray(num_branches)
        assert num_branches.shape == (self.B,)
        for s in range(self.B):
            if self.cur_parallel[s]:
                assert int(num_branches[s]) == len(self.tokens_in_branch[s]), "a running stage keeps its branches"
                continue
            if int(num_branches[s]) == 0:
                self.tokens_in_branch[s] = []
                continue
            self.cur_stage[s] += 1
            self.cur_parallel[s] = True
            self.stage_first_slot[s] = len(self.pos[s])
            # position the first token of every branch takes: the number of tokens before the stage
            # (Same-Seq), or wherever the main branch's position counter stands
            self.stage_start_pos[s] = len(self.pos[s]) if self.pos_mode == "same_seq" else self.next_main_pos[s]
            self.tokens_in_branch[s] = [0] * int(num_branches[s])

    def append_parallel(self, new_len) -> StepMeta:
        """new_len[b] tokens for every branch b (global index over the batch), Eq. 4 case 2."""
        new_len = np.asarray(new_len)
        rows = []
        g = 0
        for s in range(self.B):
            for k in range(len(self.tokens_in_branch[s])):       # branch index ascending
                for _ in range(int(new_len[g])):                 # token index ascending
                    t = self.tokens_in_branch[s][k]
                    slot = self._push(s, k + 1, t, self._branch_pos(s, k, t))
                    self.tokens_in_branch[s][k] = t + 1
                    rows.append((s, g, slot))
                g += 1
        assert g == new_len.shape[0]
        cu_new = np.zeros(g + 1, dtype=np.int32)
        np.cumsum(new_len, out=cu_new[1:])
        return self._step_meta(rows, cu_new)

    def append_mixed(self, new_len_branch, new_len_main) -> StepMeta:
        """One append call over a batch in which some sequences are in a parallel stage and the others
        serial: new_len_branch[b] tokens for every open branch b (global index), new_len_main[s]
        main-branch tokens for every serial sequence s (0 for the others).  Rows are sequence-major."""
        new_len_branch = np.asarray(new_len_branch)
        new_len_main = np.asarray(new_len_main)
        assert new_len_main.shape == (self.B,)
        rows = []
        starts = []
        g = 0
        for s in range(self.B):
            if self.cur_parallel[s]:
                assert int(new_len_main[s]) == 0, "no main-branch token while branches are open"
                for k in range(len(self.tokens_in_branch[s])):
                    starts.append(len(rows))
                    for _ in range(int(new_len_branch[g])):
                        t = self.tokens_in_branch[s][k]
                        slot = self._push(s, k + 1, t, self._branch_pos(s, k, t))
                        self.tokens_in_branch[s][k] = t + 1
                        rows.append((s, g, slot))
                    g += 1
            else:
                for _ in range(int(new_len_main[s])):
                    rows.append((s, -1, self._push_main(s)))
        assert g == new_len_branch.shape[0]
        cu_new = np.array(starts + [len(rows)], dtype=np.int32)   # first packed row of every branch, then NQ
        return self._step_meta(rows, cu_new)

    def merge(self, which=None) -> None:
        """All branches done: back to one main branch.  Nothing in the cache moves.
        `which` (bool per sequence) merges only some of the sequences; None merges all."""
        for s in range(self.B):
            if which is not None and not bool(which[s]):
                continue
            if self.cur_parallel[s]:
                if self.pos_mode == "same_max":
                    # right after the largest position a branch reached; a stage without a token reached none
                    self.next_main_pos[s] = self.stage_start_pos[s] + max(self.tokens_in_branch[s])
                elif self.fix_n:
                    # the K intervals were allotted when the stage opened ("pre-allocated", Sec. 4.5.3):
                    # they are spent whether or not a branch ever produced a token
                    self.next_main_pos[s] = self.stage_start_pos[s] + len(self.tokens_in_branch[s]) * self.fix_n
                else:
                    self.next_main_pos[s] = len(self.pos[s])
                self.cur_parallel[s] = False
                self.cur_stage[s] += 1
                self.tokens_in_branch[s] = []
                self.stage_first_slot[s] = len(self.pos[s])

    # ------------------------------------------------------------------ views
    def seq_len(self) -> np.ndarray:
        return np.array([len(p) for p in self.pos], dtype=np.int32)

    def stage_base(self) -> np.ndarray:
        """Number of leading slots that every current query may see: the first slot of the
        running parallel stage, or everything when the sequence is serial."""
        return np.array([self.stage_first_slot[s] if self.cur_parallel[s] else len(self.pos[s])
                         for s in range(self.B)], dtype=np.int32)

    def branch_len(self) -> np.ndarray:
        out = [n for s in range(self.B) for n in self.tokens_in_branch[s]]
        return np.array(out, dtype=np.int32)

    def slot_owner(self, stride: int) -> np.ndarray:
        """[B][stride] uint8: branch id (1..K) of every slot of the running parallel stage, 0 elsewhere."""
        out = np.zeros((self.B, stride), dtype=np.uint8)
        for s in range(self.B):
            if self.cur_parallel[s]:
                for slot in range(self.stage_first_slot[s], len(self.pos[s])):
                    out[s, slot] = self.branch[s][slot]
        return out

    def physical_slot(self, s: int, slot: int) -> int:
        blk = int(self.block_tables[s, slot // self.block_size])
        assert blk >= 0, "sequence outgrew its block table"
        return blk * self.block_size + slot % self.block_size

    def physical_slots(self, s: int) -> np.ndarray:
        return np.array([self.physical_slot(s, j) for j in range(len(self.pos[s]))], dtype=np.int64)

    # ------------------------------------------------------------------ mask (Eq. 2-3)
    def visible_pair(self, s: int, i: int, j: int) -> bool:
        """Eq. 2 with Eq. 3, for query slot i and key slot j of sequence s, one pair at a time."""
        bi, bj = self.branch[s][i], self.branch[s][j]
        si, sj = self.stage[s][i], self.stage[s][j]
        if bi == MAIN:                       # Eq. 3 case 1: the main branch sees every branch
            S = 1
        elif si == sj and bi == bj:          # case 2: same parallel branch
            S = 1
        elif si != sj:                       # case 3: different stage
            S = 1
        else:
            S = 0
        return S == 1 and (self.pos[s][i] > self.pos[s][j] or i == j)

    def dense_mask(self, s: int, query_slots, shared: bool = False) -> np.ndarray:
        """bool [len(query_slots)][T_s]: the same rule as visible_pair, on whole arrays.
        shared: the "Shared" mask the paper's ablation compares against (Sec. 4.5.2), read here as ordinary
        causal attention over the one cache: every token sees every slot up to and including its own,
        sibling branches included."""
        q = np.asarray(query_slots, dtype=np.int64)
        if shared:
            return np.arange(len(self.pos[s]), dtype=np.int64)[None, :] <= q[:, None]
        stage = np.asarray(self.stage[s], dtype=np.int64)
        branch = np.asarray(self.branch[s], dtype=np.int64)
        pos = np.asarray(self.pos[s], dtype=np.int64)
        slots = np.arange(len(pos), dtype=np.int64)
        q_main = (branch[q] == MAIN)[:, None]
        same_stage = stage[q][:, None] == stage[None, :]
        same_branch = branch[q][:, None] == branch[None, :]
        S = q_main | (same_stage & same_branch) | ~same_stage
        before = pos[q][:, None] > pos[None, :]
        itself = q[:, None] == slots[None, :]
        return S & (before | itself)

    def all_tokens_meta(self) -> StepMeta:
        """Every token now in the table as a query row, sequence-major in slot order: what a teacher-forced
        pass over whole sequences attends (Fig. 5, training arrangement).  q_branch holds the token's branch
        number within its own stage minus one (-1 for main-branch tokens); cu_new is not meaningful here."""
        rows = [(s, self.branch[s][j] - 1, j) for s in range(self.B) for j in range(len(self.pos[s]))]
        return self._step_meta(rows, np.zeros(1, dtype=np.int32))

    # ------------------------------------------------------------------ internals
    def _step_meta(self, rows, cu_new) -> StepMeta:
        nq = len(rows)
        q_seq = np.array([r[0] for r in rows], dtype=np.int32).reshape(nq)
        q_branch = np.array([r[1] for r in rows], dtype=np.int32).reshape(nq)
        slot = np.array([r[2] for r in rows], dtype=np.int32).reshape(nq)
        position_ids = np.array([self.pos[s][j] for s, _, j in rows], dtype=np.int32).reshape(nq)
        slot_mapping = np.array([self.physical_slot(s, j) for s, _, j in rows], dtype=np.int64).reshape(nq)
        kv_len = np.zeros(nq, dtype=np.int32)
        cu_seq_new = np.zeros(self.B + 1, dtype=np.int32)
        for s in range(self.B):
            idx = np.nonzero(q_seq == s)[0]
            cu_seq_new[s + 1] = cu_seq_new[s] + idx.size
            if idx.size:
                kv_len[idx] = self.dense_mask(s, slot[idx]).sum(axis=1)
        return StepMeta(cu_new=cu_new, cu_seq_new=cu_seq_new, q_seq=q_seq, q_branch=q_branch,
                        position_ids=position_ids, logical_slot=slot, slot_mapping=slot_mapping,
                        kv_len=kv_len)
