"""The host state machine of the Hybrid Decoding Engine (Sec. 3.3) and the sampling rule (Sec. 4.1), on the
CPU: a scripted token stream drives the engine, the oracle's token table stands behind the driver interface
and checks what the engine asks of the library."""
import numpy as np
import pytest

from engine_drive import OracleDriver, ScriptedModel
from paper_2508_08895_amd.engine import HybridEngine, SpecialTokens, filtered_distribution, sample_token

SP = SpecialTokens(title_open=901, title_close=902, branch_open=903, branch_close=904, para_open=905, para_close=906,
                   eos=999, prefix_sep=(907,))
T1, T2, T3 = [11, 12], [21], [31, 32, 33]


def _run(engine, model, prompts):
    kinds = []
    plan = engine.prefill(prompts)
    while plan is not None:
        kinds.append((plan.attention, plan.NQ))
        engine.accept(model(engine, plan))
        plan = engine.next_step()
    return kinds


def test_one_sequence_one_stage_matches_the_hand_derived_arrangement():
    """Prompt p p p; the model writes two titles and <Para>; branch 1 decodes x1 x2 </Branch>, branch 2
    y1 </Branch>; after the merge </Para>, then c and <eos>.  Expected cache order, worked out by hand from
    Sec. 3.3 and the append order (a chunk lays each branch's prefix contiguously, decode steps interleave):"""
    drv = OracleDriver(np.arange(8, dtype=np.int32)[None, :])
    eng = HybridEngine(drv, SP, batch=1)
    main = [SP.title_open, *T1, SP.title_close, SP.title_open, *T2, SP.title_close, SP.para_open, 50, SP.eos]
    model = ScriptedModel([main], [[[[61, 62, SP.branch_close], [71, SP.branch_close]]]])
    kinds = _run(eng, model, [[1, 2, 3]])
    want = [(0, 1), (0, 2), (0, 3),
            (0, SP.title_open), (0, 11), (0, 12), (0, SP.title_close), (0, SP.title_open), (0, 21), (0, SP.title_close),
            (0, SP.para_open),
            (1, SP.branch_open), (1, 11), (1, 12), (1, 907), (2, SP.branch_open), (2, 21), (2, 907),   # forced prefixes, one chunk
            (1, 61), (2, 71), (1, 62), (2, SP.branch_close), (1, SP.branch_close),                     # interleaved decode steps
            (0, SP.para_close), (0, 50), (0, SP.eos)]
    assert eng.sequence(0) == want
    assert eng.finished()
    tt = drv.tt
    assert tt.branch[0] == [b for b, _ in want]
    # positions: main tokens count everything before them; branches share positions at equal depth (Eq. 4)
    pos = tt.pos[0]
    assert pos[:11] == list(range(11))
    assert pos[11:15] == [11, 12, 13, 14] and pos[15:18] == [11, 12, 13]
    assert pos[18:23] == [15, 14, 16, 15, 17]
    assert pos[23:] == [23, 24, 25]
    # the calls: prefill and serial steps, one chunk for the prefixes, parallel-decode steps, serial again
    assert kinds[0] == ("aspd_attn_serial_decode", 3)
    assert ("aspd_attn_branch_chunk", 7) in kinds
    assert kinds.count(("aspd_attn_parallel_decode", 2)) == 2 and ("aspd_attn_parallel_decode", 1) in kinds
    assert kinds[-1] == ("aspd_attn_serial_decode", 1)
    ops = [c[0] for c in drv.calls]
    assert ops.count("merge") == 1 and ops.count("renumber") == 2
    # no branch token ever saw a sibling: the oracle's mask over the final table
    m = tt.dense_mask(0, range(len(pos)))
    for i, (bi, _) in enumerate(want):
        for j, (bj, _) in enumerate(want):
            if bi and bj and bi != bj:
                assert not m[i, j]
    assert m[23][:24].all() and not m[23][24:].any()     # </Para>, a main-branch token, sees the complete history before it


def test_batch_switches_independently_and_runs_two_rounds():
    """Three sequences: one never parallelises, one runs two parallel stages, one a stage of three branches;
    they open and end their stages at different steps of the same batch."""
    B = 3
    drv = OracleDriver(np.arange(B * 16, dtype=np.int32).reshape(B, 16))
    eng = HybridEngine(drv, SP, batch=B)

    def titles(*ts):
        out = []
        for t in ts:
            out += [SP.title_open, *t, SP.title_close]
        return out + [SP.para_open]

    main = [[40, 41, 42, 43, 44, 45, 46, SP.eos],
            [*titles(T1, T2), 51, *titles(T3, T1), 52, SP.eos],
            [60, 61, 62, *titles(T1, T2, T3), 63, 64, SP.eos]]
    stages = [[],
              [[[1, 2, 3, SP.branch_close], [4, SP.branch_close]], [[5, SP.branch_close], [6, 7, SP.branch_close]]],
              [[[8, SP.branch_close], [9, 9, 9, 9, 9, SP.branch_close], [SP.branch_close]]]]
    model = ScriptedModel(main, stages)
    kinds = _run(eng, model, [[1], [2, 2], [3, 3, 3]])
    assert eng.finished() and all(not m for m in model.main)
    assert all(not b for seq in model.stages for st in seq for b in st)
    assert [s.stages for s in eng.seqs] == [0, 2, 1]
    tt = drv.tt
    for s in range(B):
        flat = eng.sequence(s)
        assert tt.branch[s] == [b for b, _ in flat]
        # main-branch positions equal the flattened index (Eq. 4 case 1)
        for j, (b, _) in enumerate(flat):
            if b == 0:
                assert tt.pos[s][j] == j
        # every </Para> follows a stage whose branches all ended with </Branch>
        toks = [t for _, t in flat]
        assert toks.count(SP.para_close) == eng.seqs[s].stages == toks.count(SP.para_open)
    assert any(k == "aspd_attn_branch_chunk" for k, _ in kinds)
    # a step that served a serial sequence and branches of another at once went through the MIXED stage
    assert any(c[0] == "mixed" and sum(c[1]) > 0 and sum(c[2]) > 0 for c in drv.calls)
    # The same sequences as whole-sequence layouts (what a re-prefill takes): the branches of a stage one after the
    # other instead of interleaved.  Replayed through the oracle, every token gets the position it was decoded at
    # and sees the same tokens (Eq. 2-4 do not depend on the arrangement).
    from oracle.sequence_layout import replay_layout
    layouts, toks = zip(*(eng.layout(s) for s in range(B)))
    assert [r for r in layouts[0]] == [(0, len(eng.sequence(0)))]
    assert [b for b, _ in layouts[1]] == [0, 1, 2, 0, 1, 2, 0]
    assert [b for b, _ in layouts[2]] == [0, 1, 2, 3, 0]
    t2, meta = replay_layout(np.arange(B * 16, dtype=np.int32).reshape(B, 16), 16, list(layouts))
    for s in range(B):
        flat = eng.sequence(s)
        assert sorted(toks[s]) == sorted(t for _, t in flat) and sum(n for _, n in layouts[s]) == len(flat)
        # match the tokens of the two arrangements by (stage, branch, index within the branch)
        key_dec = {(tt.stage[s][j], tt.branch[s][j], tt.index_in_branch[s][j]): j for j in range(len(flat))}
        key_re = {(t2.stage[s][j], t2.branch[s][j], t2.index_in_branch[s][j]): j for j in range(len(flat))}
        assert key_dec.keys() == key_re.keys()
        m_dec = tt.dense_mask(s, np.arange(len(flat)))
        m_re = t2.dense_mask(s, np.arange(len(flat)))
        for k, jd in key_dec.items():
            jr = key_re[k]
            assert flat[jd][1] == toks[s][jr]
            assert tt.pos[s][jd] == t2.pos[s][jr]
            seen_dec = {kk for kk, j in key_dec.items() if m_dec[jd, j]}
            seen_re = {kk for kk, j in key_re.items() if m_re[jr, j]}
            assert seen_dec == seen_re, (s, k)


def test_token_budget_closes_branches_and_ends_the_sequence():
    drv = OracleDriver(np.arange(16, dtype=np.int32)[None, :])
    eng = HybridEngine(drv, SP, batch=1, max_tokens=14)
    main = [SP.title_open, *T1, SP.title_close, SP.title_open, *T2, SP.title_close, SP.para_open] + [77] * 50
    model = ScriptedModel([main], [[[[5] * 50, [6] * 50]]])
    _run(eng, model, [[1]])
    assert eng.finished()
    toks = [t for _, t in eng.sequence(0)]
    assert toks.count(SP.branch_close) == 2 and toks[-1] == SP.para_close


# ----------------------------------------------------------------------------------------- sampling (Sec. 4.1)
def test_filtered_distribution_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.normal(size=200) * 3
    p = filtered_distribution(x, temperature=0.7, top_k=20, top_p=0.8)
    assert abs(p.sum() - 1) < 1e-12 and (p >= 0).all()
    kept = np.nonzero(p)[0]
    assert 1 <= kept.size <= 20
    soft = np.exp(x / 0.7 - (x / 0.7).max())
    soft /= soft.sum()
    top20 = np.argsort(-soft)[:20]
    assert set(kept) <= set(top20.tolist())                       # top-k
    q = soft[top20] / soft[top20].sum()
    c = np.cumsum(q)
    n_keep = int(np.searchsorted(c, 0.8)) + 1                     # smallest prefix whose mass reaches top_p
    assert kept.size == n_keep and set(kept) == set(top20[:n_keep].tolist())
    assert np.allclose(p[top20[:n_keep]], q[:n_keep] / q[:n_keep].sum())   # renormalised, ratios of the softmax kept
    # invariances and limits
    assert np.allclose(filtered_distribution(x + 5.0), filtered_distribution(x))
    g = filtered_distribution(x, temperature=0.0)
    assert g[np.argmax(x)] == 1.0 and g.sum() == 1.0
    assert np.count_nonzero(filtered_distribution(x, top_k=1)) == 1
    full = filtered_distribution(x, temperature=1.0, top_k=0, top_p=1.0)
    ref = np.exp(x - x.max())
    assert np.allclose(full, ref / ref.sum())
    # one dominant token: top-p keeps it alone
    y = np.zeros(50)
    y[7] = 30.0
    assert np.count_nonzero(filtered_distribution(y)) == 1


def test_sample_token_draws_from_the_filtered_distribution():
    rng = np.random.default_rng(1)
    x = np.array([2.0, 1.5, 1.0, 0.2, -1.0, -3.0])
    p = filtered_distribution(x, temperature=0.7, top_k=4, top_p=0.9)
    draws = np.array([sample_token(x, rng, 0.7, 4, 0.9) for _ in range(20000)])
    freq = np.bincount(draws, minlength=6) / draws.size
    assert (freq[p == 0] == 0).all()
    assert np.abs(freq - p).max() < 0.015
