"""Pins for the oracle's token table: position ids (Eq. 4), cache slots, mask (Eq. 2-3).

None of these re-types the oracle's own formula: they use the hand-derived fixture, an
independently written visible-set enumeration, closed forms and invariants."""
import itertools
import os

import numpy as np
import pytest

import aspd_workloads as W
from oracle import TokenTable, MAIN
from oracle_drive import table_at, table_with_prefix


# ----------------------------------------------------------------------------- fixture
def _parse_examples(path):
    examples, cur = {}, None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        w = line.split()
        if w[0] == "example":
            cur = {"history": [], "slots": []}
            examples[w[1]] = cur
        elif w[0] == "history":
            cur["history"].append((w[1], [int(x) for x in w[2:]]))
        elif w[0] == "owners":    # owner tags of slots first .. as they stand after the history so far
            i = w.index(":")
            cur["history"].append(("owners", [int(w[1])] + [int(x) for x in w[i + 1:]]))
        elif w[0] == "slot":
            i = w.index(":")
            slot, branch, stage, pos = (int(x) for x in w[1:i])
            cur["slots"].append((slot, branch, stage, pos, {int(x) for x in w[i + 1:]}))
    return examples


def _replay(history, blocks=8):
    tt = TokenTable(np.arange(blocks, dtype=np.int32)[None, :], 16)
    metas = []
    for op, args in history:
        if op == "serial":
            metas.append(tt.append_serial([args[0]]))
        elif op == "open":
            tt.open_parallel([args[0]])
        elif op == "step":
            metas.append(tt.append_parallel(args))
        elif op == "merge":
            tt.merge()
        elif op == "owners":
            first, tags = args[0], args[1:]
            row = tt.slot_owner(16 * blocks)[0]
            assert row[first:first + len(tags)].tolist() == tags, (row[:first + len(tags)], tags)
            assert not row[:first].any() and not row[first + len(tags):].any()
            assert int(tt.stage_base()[0]) == (first if tags else len(tt.pos[0]))
    return tt, metas


@pytest.mark.parametrize("name", ["two_branches_then_merge", "two_rounds", "chunk_then_step"])
def test_worked_examples(golden_dir, name):
    ex = _parse_examples(os.path.join(golden_dir, "worked_examples.txt"))[name]
    tt, metas = _replay(ex["history"])
    T = len(ex["slots"])
    assert len(tt.pos[0]) == T
    kv_len = np.concatenate([m.kv_len for m in metas])
    slots = np.concatenate([m.logical_slot for m in metas])
    pos = np.concatenate([m.position_ids for m in metas])
    for slot, branch, stage, p, vis in ex["slots"]:
        assert tt.branch[0][slot] == branch
        assert tt.stage[0][slot] == stage
        assert tt.pos[0][slot] == p
        assert slots[slot] == slot and pos[slot] == p
        # visibility as of the moment the token was appended == as of now, restricted to then-existing
        got = {j for j in range(T) if tt.visible_pair(0, slot, j)}
        assert got == vis, (slot, got, vis)
        assert set(np.nonzero(tt.dense_mask(0, [slot])[0])[0]) == vis
        assert kv_len[slot] == len(vis)


def test_mixed_batch_worked_example(golden_dir):
    """Sequences of one batch switch stages independently: hand-derived rows and final tables."""
    tt = TokenTable(np.arange(16, dtype=np.int32).reshape(2, 8), 16)
    meta, rows, slots = None, [], []

    def check_rows():
        if meta is None:
            return
        got = list(zip(meta.q_seq.tolist(), meta.q_branch.tolist(), meta.logical_slot.tolist(),
                       meta.position_ids.tolist(), meta.kv_len.tolist()))
        assert got == rows, (got, rows)

    for line in open(os.path.join(golden_dir, "mixed_batch_example.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        w = line.split()
        if w[0] == "call":
            check_rows()
            meta, rows = None, []
            if w[1] == "serial":
                meta = tt.append_serial([int(x) for x in w[2:]])
            elif w[1] == "open":
                tt.open_parallel([int(x) for x in w[2:]])
            elif w[1] == "merge":
                tt.merge([int(x) for x in w[2:]])
            elif w[1] == "mixed":
                bar = w.index("|")
                meta = tt.append_mixed([int(x) for x in w[2:bar]], [int(x) for x in w[bar + 1:]])
        elif w[0] == "row":
            rows.append(tuple(int(x) for x in w[1:]))
        elif w[0] == "slot":
            i = w.index(":")
            slots.append(tuple(int(x) for x in w[1:i]) + ({int(x) for x in w[i + 1:]},))
    check_rows()
    assert [len(p) for p in tt.pos] == [6, 6]
    for s, slot, branch, stage, pos, vis in slots:
        assert (tt.branch[s][slot], tt.stage[s][slot], tt.pos[s][slot]) == (branch, stage, pos), (s, slot)
        assert {j for j in range(len(tt.pos[s])) if tt.visible_pair(s, slot, j)} == vis, (s, slot)
        assert set(np.nonzero(tt.dense_mask(s, [slot])[0])[0]) == vis
    assert tt.stage_base().tolist() == [6, 2] and tt.branch_len().tolist() == [1, 1, 2]


def test_mixed_batch_equals_sequences_alone():
    """Sequences do not interact: a batch driven through mixed calls, with stages opening and ending
    at different times, gives each sequence what it gets alone through the single-mode calls."""
    rng = np.random.default_rng(11)
    B = 5
    batch = TokenTable(np.arange(B * 8, dtype=np.int32).reshape(B, 8), 16)
    alone = [TokenTable(np.arange(8, dtype=np.int32)[None, :] + 8 * s, 16) for s in range(B)]
    start = rng.integers(1, 4, size=B)
    batch.append_serial(start)
    for s in range(B):
        alone[s].append_serial([start[s]])
    K = [0] * B                        # open branches per sequence
    for step in range(14):
        # some serial sequences open a stage, some running stages end
        opening = [K[s] == 0 and rng.random() < 0.4 for s in range(B)]
        ending = [K[s] > 0 and rng.random() < 0.25 for s in range(B)]
        if any(ending):
            batch.merge(ending)
            for s in range(B):
                if ending[s]:
                    alone[s].merge()
                    K[s] = 0
        if any(opening):
            for s in range(B):
                if opening[s]:
                    K[s] = int(rng.integers(1, 4))
                    alone[s].open_parallel([K[s]])
            batch.open_parallel(K)
        nb = [rng.integers(0, 3, size=K[s]) for s in range(B)]
        nm = [int(rng.integers(0, 3)) if K[s] == 0 else 0 for s in range(B)]
        meta = batch.append_mixed(np.concatenate(nb + [np.zeros(0, dtype=np.int64)]), nm)
        row = 0
        g0 = 0
        for s in range(B):
            m1 = alone[s].append_parallel(nb[s]) if K[s] else alone[s].append_serial([nm[s]])
            n = m1.NQ
            sl = slice(row, row + n)
            assert meta.q_seq[sl].tolist() == [s] * n
            assert meta.logical_slot[sl].tolist() == m1.logical_slot.tolist()
            assert meta.position_ids[sl].tolist() == m1.position_ids.tolist()
            assert meta.kv_len[sl].tolist() == m1.kv_len.tolist()
            assert meta.slot_mapping[sl].tolist() == m1.slot_mapping.tolist()
            want_branch = [b + g0 if b >= 0 else -1 for b in m1.q_branch.tolist()]
            assert meta.q_branch[sl].tolist() == want_branch
            assert meta.cu_seq_new[s] == row
            row += n
            g0 += K[s]
        assert meta.NQ == row and meta.cu_new[-1] == row
    for s in range(B):
        assert batch.pos[s] == alone[s].pos[0] and batch.branch[s] == alone[s].branch[0]
        assert batch.stage[s] == alone[s].stage[0]
        T = len(batch.pos[s])
        assert (batch.dense_mask(s, range(T)) == alone[s].dense_mask(0, range(T))).all()
    assert batch.stage_base().tolist() == [int(a.stage_base()[0]) for a in alone]


def _paradigm_history(tt):
    tt.append_serial([2])
    tt.open_parallel([2])
    for step in ([1, 1], [1, 0], [1, 0]):
        tt.append_parallel(step)
    tt.merge()
    tt.append_serial([2])
    tt.open_parallel([2])
    return tt.append_parallel([1, 1])


def _empty_stage_history(tt):
    """A stage that ends before any branch produced a token, then a main token and a second stage."""
    tt.append_serial([2])
    tt.open_parallel([2])
    tt.merge()
    tt.append_serial([1])
    tt.open_parallel([2])
    return tt.append_parallel([1, 1])


def test_position_paradigms_worked_example(golden_dir):
    seen = 0
    for line in open(os.path.join(golden_dir, "position_paradigms.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        name, want = line.split("|")
        w = name.split()
        history = _paradigm_history
        if w[0] == "empty":
            history, w = _empty_stage_history, w[1:]
        mode = (w[0], int(w[1])) if w[0] == "fix" else w[0]
        tt = TokenTable(np.arange(8, dtype=np.int32)[None, :], 16, pos_mode=mode)
        meta = history(tt)
        T = len(tt.pos[0])
        assert tt.pos[0] == [int(x) for x in want.split()], (mode, tt.pos[0])
        assert meta.position_ids.tolist() == tt.pos[0][T - 2:T]
        # what a token may see does not depend on the paradigm: the same sets as under Eq. 4
        ref = TokenTable(np.arange(8, dtype=np.int32)[None, :], 16)
        history(ref)
        assert (tt.dense_mask(0, range(T)) == ref.dense_mask(0, range(T))).all()
        seen += 1
    assert seen == 6


def test_position_paradigms_properties():
    """Same-Max: one branch makes it Same-Seq; with equal branch lengths K the main branch continues
    (K - 1) * len earlier than under Same-Seq.  Fix-N: positions of a branch are consecutive inside its
    own interval and intervals of different branches never overlap."""
    rng = np.random.default_rng(5)
    for trial in range(20):
        K = int(rng.integers(1, 5))
        lens = rng.integers(1, 6, size=K)
        pre = int(rng.integers(1, 7))
        tabs = {m: TokenTable(np.arange(8, dtype=np.int32)[None, :], 16, pos_mode=m)
                for m in ("same_seq", "same_max", ("fix", 8))}
        for m, tt in tabs.items():
            tt.append_serial([pre])
            tt.open_parallel([K])
            for new_len in W.interleaved_history(lens):
                tt.append_parallel(new_len)
            tt.merge()
            tt.append_serial([1])
        T = pre + int(lens.sum())
        assert tabs["same_seq"].pos[0][-1] == T
        assert tabs["same_max"].pos[0][-1] == pre + int(lens.max())
        if K == 1:
            assert tabs["same_max"].pos[0] == tabs["same_seq"].pos[0]
        assert tabs[("fix", 8)].pos[0][-1] == pre + 8 * K
        fx = tabs[("fix", 8)]
        for k in range(K):
            mine = [fx.pos[0][j] for j in range(pre, T) if fx.branch[0][j] == k + 1]
            assert mine == list(range(pre + 8 * k, pre + 8 * k + int(lens[k])))
        assert tabs["same_max"].pos[0][:T] == tabs["same_seq"].pos[0][:T]   # inside the stage they agree


# ----------------------------------------------------------------------------- brute force
def _visible_set_by_history(stages, slot_of):
    """Independent enumeration from the prose of Sec. 3.3: a parallel token attends the tokens of
    the main branch and of earlier stages plus its own branch's earlier tokens and itself; a
    main token attends the complete history.  `stages` is a list of ("serial", n) or
    ("parallel", [n_1..n_K]) with branch tokens appended one per active branch per step."""
    order = []          # (stage index, branch, t) in append order
    for si, (kind, arg) in enumerate(stages):
        if kind == "serial":
            order += [(si, 0, t) for t in range(arg)]
        else:
            for t in range(max(arg)):
                order += [(si, k + 1, t) for k, n in enumerate(arg) if n > t]
    vis = []
    for i, (si, bi, ti) in enumerate(order):
        if bi == 0:
            vis.append(set(range(i + 1)))
        else:
            v = {j for j, (sj, bj, tj) in enumerate(order) if sj < si}
            v |= {j for j, (sj, bj, tj) in enumerate(order) if sj == si and bj == bi and tj <= ti}
            vis.append(v)
    return order, vis


def _table_from_stages(stages):
    tt = TokenTable(np.arange(8, dtype=np.int32)[None, :], 16)
    for kind, arg in stages:
        if kind == "serial":
            tt.append_serial([arg])
        else:
            tt.open_parallel([len(arg)])
            for new_len in W.interleaved_history(arg):
                tt.append_parallel(new_len)
            tt.merge()
    return tt


def test_mask_brute_force_tiny():
    count = 0
    for L in range(0, 4):
        for K in range(1, 4):
            for lens in itertools.product(range(1, 4), repeat=K):
                for tail in (0, 2):
                    stages = [("serial", L), ("parallel", list(lens)), ("serial", tail)]
                    order, vis = _visible_set_by_history(stages, None)
                    tt = _table_from_stages(stages)
                    T = len(order)
                    assert len(tt.pos[0]) == T
                    dm = tt.dense_mask(0, np.arange(T))
                    for i in range(T):
                        got = {j for j in range(T) if tt.visible_pair(0, i, j)}
                        assert got == vis[i], (stages, i)
                        assert set(np.nonzero(dm[i])[0]) == vis[i]
                    count += 1
    assert count > 150


def test_mask_brute_force_two_rounds():
    for a, b in itertools.product([[1, 2], [3, 1, 2]], [[2], [1, 3]]):
        stages = [("serial", 2), ("parallel", a), ("serial", 1), ("parallel", b), ("serial", 1)]
        order, vis = _visible_set_by_history(stages, None)
        tt = _table_from_stages(stages)
        dm = tt.dense_mask(0, np.arange(len(order)))
        for i in range(len(order)):
            assert set(np.nonzero(dm[i])[0]) == vis[i]


# ----------------------------------------------------------------------------- closed forms
def test_parallel_counts_and_positions_closed_form():
    wl = W.random_small(11, batch=4)
    tt = table_with_prefix(wl)
    tt.open_parallel(wl.num_branches)
    cu = wl.cu_branches
    n = np.zeros(wl.NB, dtype=np.int64)
    seq_of_branch = np.repeat(np.arange(wl.B), wl.num_branches)
    for new_len in W.interleaved_history(wl.branch_len):
        m = tt.append_parallel(new_len)
        n += new_len
        active = np.nonzero(new_len)[0]
        assert m.NQ == active.size
        assert np.array_equal(m.q_branch, active)
        assert np.array_equal(m.q_seq, seq_of_branch[active])
        L = wl.prefix_len[m.q_seq]
        # number of visible keys: shared prefix plus the own branch, itself included
        assert np.array_equal(m.kv_len, L + n[active])
        # Eq. 4 case 2: stage_start + index within the branch; equal for branches at equal index
        assert np.array_equal(m.position_ids, L + n[active] - 1)
    T = wl.prefix_len + np.add.reduceat(wl.branch_len, cu[:-1])
    assert np.array_equal(tt.seq_len(), T)
    assert np.array_equal(tt.stage_base(), wl.prefix_len)
    assert np.array_equal(tt.branch_len(), wl.branch_len)
    # after the merge the first main token sits at its flattened index and sees everything
    tt.merge()
    m = tt.append_serial(np.ones(wl.B, dtype=np.int32))
    assert np.array_equal(m.position_ids, T)
    assert np.array_equal(m.kv_len, T + 1)
    assert np.array_equal(m.q_branch, -np.ones(wl.B, dtype=np.int32))
    assert np.array_equal(tt.stage_base(), T + 1)


def test_chunk_counts_closed_form():
    wl = W.random_small(12, batch=3)
    tt = table_at(wl, wl.branch_len)
    c = np.arange(wl.NB, dtype=np.int32) % 4 + 1          # ragged chunk lengths 1..4
    m = tt.append_parallel(c)
    assert m.NQ == int(c.sum())
    seq_of_branch = np.repeat(np.arange(wl.B), wl.num_branches)
    row = 0
    for b in range(wl.NB):
        assert m.cu_new[b] == row
        for j in range(c[b]):
            L = wl.prefix_len[seq_of_branch[b]]
            assert m.q_branch[row] == b
            assert m.kv_len[row] == L + wl.branch_len[b] + j + 1
            assert m.position_ids[row] == L + wl.branch_len[b] + j
            row += 1
    # the chunk of one branch occupies consecutive slots
    for b in range(wl.NB):
        sl = m.logical_slot[m.cu_new[b]:m.cu_new[b + 1]]
        assert np.array_equal(sl, sl[0] + np.arange(c[b]))


def test_single_branch_is_native_autoregression():
    # K = 1: position id == slot, every earlier token visible (Sec. 3.2, "consistent with native
    # autoregressive generation")
    wl = W.random_small(13, batch=2, branches_range=(1, 1))
    tt = table_at(wl, wl.branch_len)
    for s in range(wl.B):
        T = len(tt.pos[s])
        assert tt.pos[s] == list(range(T))
        dm = tt.dense_mask(s, np.arange(T))
        assert np.array_equal(dm, np.tril(np.ones((T, T), dtype=bool)))


def test_positions_increase_along_every_visible_chain():
    wl = W.random_small(14, batch=3)
    tt = table_at(wl, wl.branch_len)
    tt.merge()
    tt.append_serial(np.full(wl.B, 2, dtype=np.int32))
    for s in range(wl.B):
        T = len(tt.pos[s])
        dm = tt.dense_mask(s, np.arange(T))
        pos = np.array(tt.pos[s])
        for i in range(T):
            others = np.nonzero(dm[i])[0]
            others = others[others != i]
            assert np.all(pos[others] < pos[i])
            assert dm[i, i]


# ----------------------------------------------------------------------------- slots
def test_slot_mapping_bijection_and_owner_histogram():
    wl = W.random_small(15, batch=5)
    tt = table_with_prefix(wl)
    tt.open_parallel(wl.num_branches)
    seen = {}
    for new_len in W.interleaved_history(wl.branch_len):
        m = tt.append_parallel(new_len)
        for r in range(m.NQ):
            s, ls, ph = int(m.q_seq[r]), int(m.logical_slot[r]), int(m.slot_mapping[r])
            assert ph == int(wl.block_tables[s, ls // 16]) * 16 + ls % 16
            assert ph not in seen
            seen[ph] = (s, ls)
    stride = wl.max_blocks_per_seq * 16
    owner = tt.slot_owner(stride)
    cu = wl.cu_branches
    for s in range(wl.B):
        L = wl.prefix_len[s]
        tags = owner[s, L:tt.seq_len()[s]]
        hist = np.bincount(tags, minlength=wl.num_branches[s] + 1)
        assert hist[0] == 0
        assert np.array_equal(hist[1:], wl.branch_len[cu[s]:cu[s + 1]])
        assert not owner[s, :L].any() and not owner[s, tt.seq_len()[s]:].any()
    # all physical slots of all sequences are distinct
    allp = np.concatenate([tt.physical_slots(s) for s in range(wl.B)])
    assert np.unique(allp).size == allp.size


def test_identity_table_slot_mapping():
    wl = W.config(1)
    tt = table_at(wl, wl.branch_len)
    assert np.array_equal(tt.physical_slots(0), np.arange(94))
    assert tt.pos[0][-3:] != []  # table non-empty
    # config 1: the three last-appended branch tokens sit at positions 64+4, 64+8, 64+15
    last = {}
    for slot in range(64, 94):
        last[tt.branch[0][slot]] = tt.pos[0][slot]
    assert last == {1: 68, 2: 72, 3: 79}


def test_replay_is_deterministic():
    wl = W.random_small(16, batch=3)
    a, b = table_at(wl, wl.branch_len), table_at(wl, wl.branch_len)
    assert a.pos == b.pos and a.branch == b.branch and a.stage == b.stage


# ----------------------------------------------------------------------------- shared mask of the ablation
def test_shared_mask_is_causal_attention_over_the_cache():
    """The ablation's "Shared" mask: lower-triangular in slot order whatever the branches are; with one
    branch per stage it coincides with the branch-independent mask (which is then native autoregression);
    main-branch rows are the same under both masks."""
    wl = W.random_small(77, batch=3, branches_range=(2, 4), branch_len_range=(2, 6), prefix_range=(1, 9))
    tt = table_at(wl, wl.branch_len)
    tt.merge()
    tt.append_serial(np.ones(wl.B, dtype=np.int32))
    for s in range(wl.B):
        T = len(tt.pos[s])
        m = tt.dense_mask(s, range(T), shared=True)
        assert (m == np.tril(np.ones((T, T), dtype=bool))).all()
        ind = tt.dense_mask(s, range(T))
        main_rows = [j for j in range(T) if tt.branch[s][j] == MAIN]
        assert (m[main_rows] == ind[main_rows]).all()
        assert (m | ind == m).all()                       # the shared mask only ever adds keys
    one = W.random_small(78, batch=2, branches_range=(1, 1), branch_len_range=(3, 9), prefix_range=(2, 9))
    t1 = table_at(one, one.branch_len)
    for s in range(one.B):
        T = len(t1.pos[s])
        assert (t1.dense_mask(s, range(T), shared=True) == t1.dense_mask(s, range(T))).all()
