"""Host side of the Hybrid Decoding Engine (ASPD Sec. 3.3): the state machine that switches every
sequence of a batch between serial and parallel decoding, driven by the special tokens, and the sampling
rule of Sec. 4.1.  No attention arithmetic happens here: the engine decides which tokens the next step
appends, asks the library for their metadata (aspd_build_branch_meta and friends, through a driver
object) and tells the caller which attention entry point the step takes.  The model (embedding, projections,
MLP, logits) is the caller's.

Control flow, per sequence (Sec. 3.3):
  * serial mode: the model writes the main branch.  Titles appear between <Title> and </Title>.
  * <Para> ends the titles: a parallel stage opens with one branch per title since the last stage.
    Branch i is given the forced prefix  <Branch> title_i tokens ... prefix_sep tokens  (the paper's
    "<Branch>Ti: "), appended in one call per stage (the branch-chunk attention call).
  * every following step appends one token to every unfinished branch (parallel decode).  A branch that
    produces </Branch> is finished once that token has been appended.
  * when all branches are finished the stage is merged (no KV is touched) and </Para> is appended to the
    main branch, which goes on serially.  Stages may follow one another.
Sequences of a batch switch independently; one step serves serial and parallel sequences together (the
MIXED metadata stage).  A sequence ends at `eos` or after max_tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np


@dataclass(frozen=True)
class SpecialTokens:
    """Ids of the six tokens the vocabulary is augmented with (Sec. 3.3), plus end-of-sequence and the
    tokens of the separator that follows a title in a branch prefix (": " in the paper)."""
    title_open: int
    title_close: int
    branch_open: int
    branch_close: int
    para_open: int
    para_close: int
    eos: int
    prefix_sep: tuple = ()


# ------------------------------------------------------------------------------------------- sampling
def sample_token(logits: np.ndarray, rng: np.random.Generator, temperature: float = 0.7, top_k: int = 20,
                 top_p: float = 0.8) -> int:
    """One token id from `logits` [vocab] under the decoding settings of Sec. 4.1 (temperature 0.7, top-k 20,
    top-p 0.8), in the customary order: temperature, then the k most likely tokens, then the smallest set of
    them whose probability reaches top_p, renormalised.  temperature 0 is greedy."""
    p = filtered_distribution(logits, temperature, top_k, top_p)
    return int(rng.choice(p.shape[0], p=p))


def filtered_distribution(logits: np.ndarray, temperature: float = 0.7, top_k: int = 20, top_p: float = 0.8) -> np.ndarray:
    """The distribution sample_token draws from, float64 [vocab]."""
    x = np.asarray(logits, dtype=np.float64)
    n = x.shape[0]
    if temperature <= 0.0:
        p = np.zeros(n)
        p[int(np.argmax(x))] = 1.0
        return p
    x = x / temperature
    x = x - x.max()
    p = np.exp(x)
    p /= p.sum()
    order = np.argsort(-p, kind="stable")          # most likely first; ties by id
    keep = order[: max(1, min(int(top_k), n))] if top_k and top_k > 0 else order
    q = p[keep] / p[keep].sum()
    if top_p is not None and top_p < 1.0:
        c = np.cumsum(q)
        cut = int(np.searchsorted(c, top_p - 1e-12)) + 1   # smallest prefix whose mass reaches top_p
        keep, q = keep[:cut], q[:cut]
    out = np.zeros(n)
    out[keep] = q / q.sum()
    return out


# ------------------------------------------------------------------------------------------- engine
@dataclass
class _Branch:
    prefix: List[int]                 # forced tokens, fed by the stage's first step
    tokens: List[int] = field(default_factory=list)   # everything appended to the branch so far
    pending: Optional[int] = None     # token chosen after the last step, appended by the next
    fed: bool = False                 # the prefix has been appended
    finished: bool = False            # </Branch> has been appended


@dataclass
class _Seq:
    main: List[int] = field(default_factory=list)      # tokens appended to the main branch, in order
    flat: List[tuple] = field(default_factory=list)    # (0 = main | branch number 1.., token) in append order
    pending: List[int] = field(default_factory=list)   # main-branch tokens the next step appends
    titles: List[List[int]] = field(default_factory=list)
    in_title: Optional[List[int]] = None
    branches: List[_Branch] = field(default_factory=list)
    done: bool = False                # nothing more will be chosen for this sequence
    produced: int = 0                 # tokens chosen so far
    stages: int = 0                   # parallel stages opened so far


@dataclass
class StepPlan:
    """What one engine step appends.  Rows are packed in the library's order (sequence, then branch, then
    token); per row: the token id fed to the model, its sequence, its branch (0-based within the sequence,
    -1 = main branch) and whether the model's output for the row chooses a next token."""
    tokens: np.ndarray
    seq: np.ndarray
    branch: np.ndarray
    wants_output: np.ndarray
    attention: str                    # "aspd_attn_parallel_decode" | "aspd_attn_branch_chunk" | "aspd_attn_serial_decode"
    step: object                      # what the driver's metadata call returned (position ids, slot mapping, ...)
    max_new_per_seq: int

    @property
    def NQ(self) -> int:
        return int(self.tokens.shape[0])


class HybridEngine:
    """driver: the library's metadata calls on one batch state -
         serial(new_len[B], hint) / mixed(new_len_branch[NB], new_len_main[B], hint) -> step,
         renumber(num_branches[B]), merge(which[B]).
       LibraryDriver below wraps the HIP library; the CPU tests substitute a checker.
       Use:  plan = engine.prefill(prompts);  while plan: chosen = model(plan); engine.accept(chosen);
             plan = engine.next_step()."""

    def __init__(self, driver, special: SpecialTokens, batch: int, max_tokens: int = 1 << 30):
        self.d = driver
        self.sp = special
        self.B = int(batch)
        self.max_tokens = int(max_tokens)
        self.seqs = [_Seq() for _ in range(self.B)]
        self._last: Optional[StepPlan] = None

    def prefill(self, prompts: Sequence[Sequence[int]]) -> StepPlan:
        """The prompts as main-branch tokens of one serial step (causal among themselves).  The output of
        each sequence's last row chooses its first generated token."""
        assert len(prompts) == self.B and self._last is None
        for s, p in zip(self.seqs, prompts):
            assert len(p) > 0 and not s.main
            s.pending = list(p)
        return self.next_step()

    def finished(self) -> bool:
        return all(s.done and not s.pending and not s.branches for s in self.seqs)

    def sequence(self, s: int) -> List[tuple]:
        """(branch number, token) of sequence s in cache order: 0 = main branch, k = k-th branch of its stage."""
        return list(self.seqs[s].flat)

    def layout(self, s: int):
        """Sequence s as a whole-sequence layout in the training arrangement (Fig. 5: the branches of a stage laid
        one after the other): (runs, tokens), runs = [(0, n) main-branch tokens | (k, n) the k-th branch of a
        stage], tokens in that order.  What a re-prefill of the sequence takes (aspd_build_sequence_meta; the
        Same-Re paradigm of Sec. 4.5.3 re-prefills after every stage).  A stage ends at the next main-branch
        token, which the engine always appends after a merge."""
        runs, tokens = [], []
        stage = {}                    # branch number -> tokens, of the stage being collected

        def close():
            for k in sorted(stage):
                runs.append((k, len(stage[k])))
                tokens.extend(stage[k])
            stage.clear()

        for b, t in self.seqs[s].flat:
            if b == 0:
                close()
                if runs and runs[-1][0] == 0:
                    runs[-1] = (0, runs[-1][1] + 1)
                else:
                    runs.append((0, 1))
                tokens.append(t)
            else:
                stage.setdefault(b, []).append(t)
        close()
        return runs, tokens

    # ------------------------------------------------------------------ one step
    def next_step(self) -> Optional[StepPlan]:
        """Metadata for the tokens that are due; None when every sequence has ended."""
        assert self._last is None, "accept() the previous step's tokens first"
        sp = self.sp
        nb, nm = [], []
        toks, seq, br, want = [], [], [], []
        chunky = False
        for si, s in enumerate(self.seqs):
            if s.branches:                                   # in a parallel stage
                nm.append(0)
                for k, b in enumerate(s.branches):
                    new = list(b.prefix) if not b.fed else ([b.pending] if b.pending is not None else [])
                    nb.append(len(new))
                    chunky |= len(new) > 1
                    for i, t in enumerate(new):
                        toks.append(t)
                        seq.append(si)
                        br.append(k)
                        # the closing token of a branch is appended for the record; nothing follows it
                        want.append(i == len(new) - 1 and t != sp.branch_close)
            else:
                new = list(s.pending)
                nm.append(len(new))
                chunky |= len(new) > 1
                opens = bool(new) and new[-1] == sp.para_open and bool(s.titles)
                for i, t in enumerate(new):
                    toks.append(t)
                    seq.append(si)
                    br.append(-1)
                    # nothing is chosen after <eos>, nor after a <Para> that opens a stage (forced prefixes follow)
                    want.append(i == len(new) - 1 and t != sp.eos and not opens and not s.done)
        if not toks:
            return None
        hint = int(np.bincount(np.asarray(seq), minlength=self.B).max())
        if nb:
            step = self.d.mixed(np.asarray(nb, dtype=np.int32), np.asarray(nm, dtype=np.int32), hint)
            attention = "aspd_attn_branch_chunk" if chunky else "aspd_attn_parallel_decode"
        else:
            step = self.d.serial(np.asarray(nm, dtype=np.int32), hint)
            attention = "aspd_attn_serial_decode"
        plan = StepPlan(np.asarray(toks, dtype=np.int64), np.asarray(seq, dtype=np.int32), np.asarray(br, dtype=np.int32),
                        np.asarray(want, dtype=bool), attention, step, hint)
        self._last = plan
        return plan

    def accept(self, next_tokens: Sequence[int]) -> None:
        """next_tokens: one token id per row of the last step whose wants_output is set, in row order (what
        the model, through sample_token, chose to follow that row).  Advances every sequence's state and
        makes the metadata calls of the stage switches that follow from it (merge, renumbering)."""
        plan = self._last
        assert plan is not None
        self._last = None
        sp = self.sp
        chosen = [int(t) for t in next_tokens]
        assert len(chosen) == int(plan.wants_output.sum())
        opening = [False] * self.B
        # 1. book what the step appended
        for si, s in enumerate(self.seqs):
            if not s.branches:
                s.pending = []
        for r in range(plan.NQ):
            si, t, k = int(plan.seq[r]), int(plan.tokens[r]), int(plan.branch[r])
            s = self.seqs[si]
            s.flat.append((k + 1 if k >= 0 else 0, t))
            if k >= 0:
                b = s.branches[k]
                b.tokens.append(t)
                b.fed = True
                b.pending = None
                b.finished |= t == sp.branch_close
            else:
                s.main.append(t)
                if t == sp.para_open and s.titles and not s.done:
                    opening[si] = True
        # 2. route the chosen tokens
        it = iter(chosen)
        for r in range(plan.NQ):
            if not plan.wants_output[r]:
                continue
            t = next(it)
            s = self.seqs[int(plan.seq[r])]
            k = int(plan.branch[r])
            s.produced += 1
            if k >= 0:
                # (a sequence that has used up its budget closes its branches)
                s.branches[k].pending = sp.branch_close if s.produced >= self.max_tokens else t
            else:
                self._main_token(s, t)
        # 3. stages that end: every branch has its </Branch> in the cache
        ending = [bool(s.branches) and all(b.finished for b in s.branches) for s in self.seqs]
        if any(ending):
            self.d.merge(np.asarray(ending, dtype=np.int32))
            for si, s in enumerate(self.seqs):
                if ending[si]:
                    s.branches = []
                    s.pending = [sp.para_close]   # Sec. 3.3: </Para> is appended, serial decoding resumes
                    if s.produced >= self.max_tokens:
                        s.done = True
        # 4. stages that open: <Para> has been appended after at least one title
        for si, s in enumerate(self.seqs):
            if opening[si]:
                s.branches = [_Branch(prefix=[sp.branch_open] + list(t) + list(sp.prefix_sep)) for t in s.titles]
                s.titles = []
                s.in_title = None
                s.pending = []
                s.stages += 1
        if any(ending) or any(opening):
            self.d.renumber(np.asarray([len(s.branches) for s in self.seqs], dtype=np.int32))

    def _main_token(self, s: _Seq, t: int) -> None:
        sp = self.sp
        s.pending = [t]
        if t == sp.eos or s.produced >= self.max_tokens:
            s.done = True        # the token is still appended by the next step, for the record; nothing follows it
        if t == sp.title_open:
            s.in_title = []
        elif t == sp.title_close:
            if s.in_title is not None:
                s.titles.append(s.in_title)
            s.in_title = None
        elif s.in_title is not None:
            s.in_title.append(t)


class LibraryDriver:
    """The HIP library behind the engine: metadata calls on one BatchState (see binding.py)."""

    def __init__(self, binding, kv, state):
        self.A, self.kv, self.state = binding, kv, state

    def _dev(self, x):
        import torch
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(self.state.device)

    def serial(self, new_len, hint):
        return self.A.aspd_build_branch_meta(self.kv, self.state, self.A.STAGE_SERIAL, self._dev(new_len),
                                             NQ=int(np.sum(new_len)), max_new_per_seq=int(hint))

    def mixed(self, new_len_branch, new_len_main, hint):
        both = np.concatenate([new_len_branch, new_len_main]).astype(np.int32)
        return self.A.aspd_build_branch_meta(self.kv, self.state, self.A.STAGE_MIXED, self._dev(both), NQ=int(both.sum()),
                                             max_new_per_seq=int(hint))

    def renumber(self, num_branches):
        import torch
        cu = np.zeros(len(num_branches) + 1, dtype=np.int32)
        np.cumsum(num_branches, out=cu[1:])
        self.A.aspd_renumber_branches(self.state, torch.from_numpy(cu))

    def merge(self, which):
        self.A.aspd_build_branch_meta(self.kv, self.state, self.A.STAGE_MERGE, self._dev(which))

    def reprefill(self, layouts):
        """Metadata of whole sequences given by their layouts (HybridEngine.layout): the step that
        aspd_rope_append and aspd_attn_full_sequence take.  Rebuilds the state of every sequence from slot 0."""
        cu = np.zeros(len(layouts) + 1, dtype=np.int32)
        np.cumsum([len(r) for r in layouts], out=cu[1:])
        br = [b for r in layouts for b, _ in r] or [0]
        ln = [n for r in layouts for _, n in r] or [0]
        nq = int(sum(n for r in layouts for _, n in r))
        return self.A.aspd_build_sequence_meta(self.kv, self.state, self._dev(cu), self._dev(br), self._dev(ln), NQ=nq)
