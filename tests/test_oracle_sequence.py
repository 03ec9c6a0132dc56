"""Pins of the oracle's whole-sequence view (oracle/sequence_layout.py, TokenTable.all_tokens_meta): the mask and
position ids of ALL tokens of a multi-stage sequence in the training arrangement of Fig. 5.  Checked against a
hand-worked example (tests/golden/whole_sequence_example.txt), against what every token saw when it was
appended (a token's visible set never changes afterwards), against an independently written rule in cache terms,
and against torch's attention with an explicit mask."""
import os

import numpy as np
import pytest
import torch

import aspd_workloads as W
from oracle import attention
from oracle.sequence_layout import replay_layout, stages_of
from oracle.token_table import TokenTable

GOLD = os.path.join(os.path.dirname(__file__), "golden", "whole_sequence_example.txt")


def _golden():
    runs, pos, vis = None, {}, {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, _, val = line.partition(":")
        if key == "runs":
            runs = [tuple(int(x) for x in r.split(":")) for r in val.split()]
        elif key.startswith("positions"):
            pos[key[len("positions "):]] = [int(x) for x in val.split()]
        elif key.startswith("visible"):
            vis[int(key.split()[1])] = [int(x) for x in val.split()]
    return runs, pos, vis


@pytest.mark.parametrize("mode", ["same_seq", "same_max", "fix 3"])
def test_hand_worked_example(mode):
    runs, pos, vis = _golden()
    pm = ("fix", 3) if mode == "fix 3" else mode
    bt = np.arange(2, dtype=np.int32).reshape(1, 2)
    tt, meta = replay_layout(bt, 16, [runs], pm)
    T = len(vis)
    assert meta.NQ == T and meta.logical_slot.tolist() == list(range(T))
    assert meta.position_ids.tolist() == pos[mode]
    mask = tt.dense_mask(0, np.arange(T))
    for i in range(T):
        assert np.nonzero(mask[i])[0].tolist() == vis[i], (mode, i)
        assert meta.kv_len[i] == len(vis[i])
    want_branch = [b - 1 for b, n in runs for _ in range(n)]
    assert meta.q_branch.tolist() == want_branch


def _cache_rule(runs):
    """The same mask from the layout alone, in cache terms: slot j is visible to slot i iff j <= i and (i is a
    main-branch token, or j lies before i's stage, or j belongs to i's branch)."""
    tag, base = [], []
    first = 0
    for b, n in runs:
        if b == 1:
            first = len(tag)
        for _ in range(n):
            base.append(first if b else len(tag))
            tag.append(b)
    T = len(tag)
    m = np.zeros((T, T), dtype=bool)
    for i in range(T):
        for j in range(i + 1):
            m[i, j] = tag[i] == 0 or j < base[i] or tag[j] == tag[i]
    return m, np.array(tag), np.array(base)


@pytest.mark.parametrize("seed", range(6))
def test_mask_equals_cache_rule_and_append_time_view(seed):
    wl = W.random_small(seed=4000 + seed, batch=3, prefix_range=(0, 40), branch_len_range=(1, 12))
    layouts = W.random_layouts(wl, seed=seed, fill=0.5)
    for pm in ("same_seq", "same_max"):
        tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts, pm)
        # what every token saw when it was appended: replay again, call by call
        t2 = TokenTable(wl.block_tables, wl.block_size, pos_mode=pm)
        stages = [stages_of(r) for r in layouts]
        seen = [dict() for _ in range(wl.B)]
        for t in range(max(len(st) for st in stages)):
            K = np.zeros(wl.B, dtype=np.int32)
            main = np.zeros(wl.B, dtype=np.int32)
            branch = []
            for s in range(wl.B):
                if t < len(stages[s]):
                    kind, what = stages[s][t]
                    if kind == "main":
                        main[s] = what
                    else:
                        K[s] = len(what)
                        branch.extend(what)
            t2.open_parallel(K)
            m = t2.append_mixed(np.array(branch, dtype=np.int32), main)
            for s in range(wl.B):
                rows = np.nonzero(m.q_seq == s)[0]
                if rows.size:
                    dm = t2.dense_mask(s, m.logical_slot[rows])
                    for r, row in zip(rows, dm):
                        seen[s][int(m.logical_slot[r])] = np.nonzero(row)[0].tolist()
            t2.merge()
        for s in range(wl.B):
            T = int(tt.seq_len()[s])
            assert T == sum(n for _, n in layouts[s])
            full = tt.dense_mask(s, np.arange(T))
            rule, tag, base = _cache_rule(layouts[s])
            assert (full == rule).all(), (seed, pm, s)
            for i in range(T):
                assert np.nonzero(full[i])[0].tolist() == seen[s][i], (seed, pm, s, i)
            rows = np.nonzero(meta.q_seq == s)[0]
            assert meta.logical_slot[rows].tolist() == list(range(T))
            assert (meta.kv_len[rows] == full.sum(axis=1)).all()
            assert (meta.q_branch[rows] == tag - 1).all()


def test_one_main_run_is_plain_causal_attention():
    wl = W.random_small(seed=4100, batch=2, num_q_heads=4, num_kv_heads=2, head_dim=64, prefix_range=(20, 40))
    T = [37, 52]
    layouts = [[(0, T[0])], [(0, T[1])]]
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    assert meta.position_ids.tolist() == list(range(T[0])) + list(range(T[1]))
    q = wl.draw_q(meta.NQ)
    out, _ = attention.attend(tt, meta, q, wl.k_cache, wl.v_cache)
    row = 0
    for s in range(2):
        phys = torch.from_numpy(tt.physical_slots(s))
        for h in range(4):
            k = wl.k_cache[phys // 16, h // 2, phys % 16].double()
            v = wl.v_cache[phys // 16, h // 2, phys % 16].double()
            ref = torch.nn.functional.scaled_dot_product_attention(q[row:row + T[s], h].double()[None], k[None], v[None],
                                                                  is_causal=True)[0]
            assert np.abs(out[row:row + T[s], h] - ref.numpy()).max() < 1e-12
        row += T[s]


def test_attention_equals_torch_with_the_cache_rule_mask():
    wl = W.random_small(seed=4200, batch=2, num_q_heads=4, num_kv_heads=2, head_dim=64, prefix_range=(10, 30),
                        branch_len_range=(4, 12))
    layouts = W.random_layouts(wl, seed=77, fill=0.6)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    q = wl.draw_q(meta.NQ)
    out, _ = attention.attend(tt, meta, q, wl.k_cache, wl.v_cache)
    row = 0
    for s in range(2):
        rule, _, _ = _cache_rule(layouts[s])
        T = rule.shape[0]
        phys = torch.from_numpy(tt.physical_slots(s))
        for h in range(4):
            k = wl.k_cache[phys // 16, h // 2, phys % 16].double()
            v = wl.v_cache[phys // 16, h // 2, phys % 16].double()
            ref = torch.nn.functional.scaled_dot_product_attention(q[row:row + T, h].double()[None], k[None], v[None],
                                                                  attn_mask=torch.from_numpy(rule)[None])[0]
            assert np.abs(out[row:row + T, h] - ref.numpy()).max() < 1e-12
        row += T


def test_bad_numbering_is_refused():
    with pytest.raises(AssertionError):
        stages_of([(0, 3), (2, 4)])
    with pytest.raises(AssertionError):
        stages_of([(1, 3), (3, 4)])
