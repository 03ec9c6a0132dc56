"""GPU parity of the whole-sequence calls (aspd_build_sequence_meta, aspd_attn_full_sequence) against the
oracle: every token of a batch of multi-stage sequences (training arrangement of Fig. 5) as a query row.
Metadata bit-exact, attention within the bf16 tolerance; the state the call leaves is checked by decoding on
from it."""
import numpy as np
import pytest
import torch

import aspd_workloads as W
from oracle import attend
from oracle.sequence_layout import replay_layout

pytestmark = pytest.mark.gpu

TOL, LSE_TOL = 2e-2, 2e-3
HDR = 16


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_08895_amd import binding
    binding.lib()
    return binding


def _layout_arrays(layouts):
    cu = np.zeros(len(layouts) + 1, dtype=np.int32)
    np.cumsum([len(r) for r in layouts], out=cu[1:])
    br = np.array([b for r in layouts for b, _ in r], dtype=np.int32)
    ln = np.array([n for r in layouts for _, n in r], dtype=np.int32)
    return cu, br, ln


def _build(A, gb, layouts, NQ=None, pos_mode=None):
    cu, br, ln = _layout_arrays(layouts)
    if pos_mode is not None:
        gb.state.pos_mode = pos_mode
    nq = int(ln.sum()) if NQ is None else NQ
    step = A.aspd_build_sequence_meta(gb.kv, gb.state, gb._dev_i32(cu), gb._dev_i32(br if br.size else np.zeros(1)),
                                      gb._dev_i32(ln if ln.size else np.zeros(1)), NQ=nq)
    torch.cuda.synchronize()
    return step


def _stage_first_slots(tt, s):
    """Per slot: the first slot of the token's stage for branch tokens, the slot itself for main-branch tokens."""
    stage, branch = tt.stage[s], tt.branch[s]
    out, first = [], {}
    for j, (st, b) in enumerate(zip(stage, branch)):
        first.setdefault(st, j)
        out.append(first[st] if b else j)
    return out


def _check_meta(A, gb, wl, step, tt, meta, layouts):
    from gpu_drive import STEP_FIELDS
    assert gb.fault() == 0
    assert step.NQ == meta.NQ
    for f in STEP_FIELDS:
        if f == "cu_new":
            continue
        got = getattr(step, f).cpu().numpy()
        want = getattr(meta, f)
        if f != "cu_seq_new":
            got = got[:meta.NQ]
        assert got.dtype == want.dtype and np.array_equal(got, want), f
    T = tt.seq_len()
    st = gb.state
    assert np.array_equal(st.seq_len.cpu().numpy(), T)
    assert np.array_equal(st.stage_base.cpu().numpy(), T)
    assert not st.stage_open.cpu().numpy().any()
    assert st.main_pos.cpu().numpy().tolist() == list(tt.next_main_pos)
    own = st.slot_owner.cpu().numpy()
    plan = step.plan.cpu().numpy().view(np.int32)
    G = wl.num_q_heads // wl.num_kv_heads
    qpg = 256 // G
    assert plan[1] == qpg and plan[2] == meta.NQ and plan[3] == wl.B
    row_base = plan[HDR:HDR + meta.NQ]
    items = plan[HDR + ((meta.NQ + 3) & ~3):][:4 * plan[0]].reshape(-1, 4)
    covered = np.zeros(meta.NQ, dtype=np.int32)
    cost = []
    for s_, q0, nq, npg in items.tolist():
        assert 0 <= s_ < wl.B and 1 <= nq <= qpg
        first = meta.cu_seq_new[s_]
        assert (q0 - first) % qpg == 0 and q0 + nq <= meta.cu_seq_new[s_ + 1]
        assert nq == qpg or q0 + nq == meta.cu_seq_new[s_ + 1]
        assert npg == (q0 - first + nq + 15) // 16
        covered[q0:q0 + nq] += 1
        cost.append(npg)
    assert (covered == 1).all()
    # longest key ranges first, up to the interleaving of sequences of different lengths: a row group is never
    # listed after one of the same sequence that is shorter
    for s in range(wl.B):
        mine = [c for (s_, *_), c in zip(items.tolist(), cost) if s_ == s]
        assert mine == sorted(mine, reverse=True)
    for s in range(wl.B):
        assert own[s, :T[s]].tolist() == list(tt.branch[s])
        r0 = meta.cu_seq_new[s]
        assert row_base[r0:r0 + T[s]].tolist() == _stage_first_slots(tt, s)


def _check_attention(A, gb, wl, step, tt, meta, rows=None, label=""):
    q = wl.draw_q(meta.NQ)
    lse = torch.full((meta.NQ, wl.num_q_heads), float("nan"), dtype=torch.float32, device=gb.dev)
    out = torch.full((meta.NQ, wl.num_q_heads, wl.head_dim), float("nan"), dtype=q.dtype, device=gb.dev)
    A.aspd_attn_full_sequence(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace, out=out, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = attend(tt, meta, q, wl.k_cache, wl.v_cache, rows=rows)
    got = out.float().cpu().numpy().astype(np.float64)
    got_lse = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), label              # every row was written, sampled or not
    sel = np.arange(meta.NQ) if rows is None else np.asarray(rows)
    err = np.abs(got[sel] - ref[sel]).max()
    lerr = np.abs(got_lse[sel] - ref_lse[sel]).max()
    print(f"[{label}] rows={sel.size} of {meta.NQ} max|out-ref|={err:.3e} max|lse-ref|={lerr:.3e}", flush=True)
    assert err <= TOL and lerr <= LSE_TOL, (label, err, lerr)
    # the counters the launch used are back at zero
    assert int(gb.workspace[:8].view(torch.int32).abs().sum().item()) == 0
    return out


@pytest.mark.parametrize("seed", range(4))
def test_small_random_layouts(A, seed):
    from gpu_drive import GpuBatch
    heads = [(32, 8, 128), (8, 4, 64), (16, 16, 128), (32, 2, 64)][seed]
    wl = W.random_small(seed=5000 + seed, num_q_heads=heads[0], num_kv_heads=heads[1], head_dim=heads[2], batch=4,
                        prefix_range=(0, 300), branches_range=(1, 6), branch_len_range=(1, 60))
    layouts = W.random_layouts(wl, seed=seed, fill=0.9)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts)
    _check_meta(A, gb, wl, step, tt, meta, layouts)
    _check_attention(A, gb, wl, step, tt, meta, label=f"small {seed} {heads}")


def test_hand_worked_example_on_the_gpu(A):
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5100, batch=1, prefix_range=(10, 10), branches_range=(2, 2), branch_len_range=(2, 2))
    runs = [(0, 2), (1, 2), (2, 1), (0, 1), (1, 1), (2, 2), (0, 1)]
    for pm_gpu, pm, want in ((A.POS_SAME_SEQ, "same_seq", [0, 1, 2, 3, 2, 5, 6, 6, 7, 9]),
                             (A.POS_SAME_MAX, "same_max", [0, 1, 2, 3, 2, 4, 5, 5, 6, 7]),
                             (A.POS_FIX_N(3), ("fix", 3), [0, 1, 2, 3, 5, 8, 9, 12, 13, 15])):
        tt, meta = replay_layout(wl.block_tables, wl.block_size, [runs], pm)
        gb = GpuBatch(wl)
        step = _build(A, gb, [runs], pos_mode=pm_gpu)
        assert step.position_ids.cpu().numpy()[:10].tolist() == want      # the paper-derived values themselves
        assert step.kv_len.cpu().numpy()[:10].tolist() == [1, 2, 3, 4, 3, 6, 7, 7, 8, 10]
        _check_meta(A, gb, wl, step, tt, meta, [runs])
        _check_attention(A, gb, wl, step, tt, meta, label=f"worked example {pm}")


@pytest.mark.parametrize("mode", ["same_max", "fix"])
def test_position_paradigms(A, mode):
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5200, batch=3, prefix_range=(0, 100), branches_range=(1, 5), branch_len_range=(1, 30))
    layouts = W.random_layouts(wl, seed=11, fill=0.8)
    longest = max([n for r in layouts for b, n in r if b > 0] + [1])
    pm, pm_gpu = ("same_max", A.POS_SAME_MAX) if mode == "same_max" else (("fix", longest), A.POS_FIX_N(longest))
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts, pm)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts, pos_mode=pm_gpu)
    _check_meta(A, gb, wl, step, tt, meta, layouts)
    _check_attention(A, gb, wl, step, tt, meta, label=f"paradigm {mode}")


def test_long_sequences_many_row_groups(A):
    """Four sequences of two to three thousand tokens (dozens of row groups each, key ranges from one page to
    two hundred), every row checked."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5300, batch=4, prefix_range=(1200, 2000), branches_range=(2, 6), branch_len_range=(60, 200),
                        extra_tokens_per_branch=0)
    layouts = W.random_layouts(wl, seed=5, max_stages=4, fill=1.0)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts)
    _check_meta(A, gb, wl, step, tt, meta, layouts)
    _check_attention(A, gb, wl, step, tt, meta, label="long")


def test_config5_sized_batch_on_sampled_rows(A):
    """A batch of the size of configuration 5 (64 sequences of 1 100 to 9 400 tokens): metadata of all 330 000
    rows bit-exact, attention on a seeded sample of rows the oracle computes one by one, and every output finite."""
    from gpu_drive import GpuBatch
    wl = W.config(5)
    layouts = W.random_layouts(wl, seed=9, max_stages=3, max_branches=10, fill=0.97)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl, poison_unmapped=False)
    step = _build(A, gb, layouts)
    _check_meta(A, gb, wl, step, tt, meta, layouts)
    rows = np.sort(np.random.default_rng(3).choice(meta.NQ, size=96, replace=False))
    _check_attention(A, gb, wl, step, tt, meta, rows=rows, label="config-5 sized")


def test_decoding_goes_on_from_the_state_the_call_leaves(A):
    """Re-prefill, then a serial step, a new parallel stage with a chunk and a decode step, a merge and a last
    serial step, each against the oracle continuing from the replayed table."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    wl = W.random_small(seed=5400, batch=3, prefix_range=(50, 200), branches_range=(2, 4), branch_len_range=(5, 30),
                        extra_tokens_per_branch=24, extra_tokens_per_seq=8)
    layouts = W.random_layouts(wl, seed=21, fill=0.55)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts)
    _check_meta(A, gb, wl, step, tt, meta, layouts)
    _check_attention(A, gb, wl, step, tt, meta, label="re-prefill")

    def compare(step, meta, fn, label):
        assert_step_equal(step, meta)
        q = wl.draw_q(meta.NQ)
        out = fn(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace)
        torch.cuda.synchronize()
        ref, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache)
        err = np.abs(out.float().cpu().numpy() - ref).max()
        print(f"[after re-prefill: {label}] max|out-ref|={err:.3e}", flush=True)
        assert err <= TOL

    one = np.ones(wl.B, dtype=np.int32)
    compare(gb.serial(one), tt.append_serial(one), A.aspd_attn_serial_decode, "serial")
    tt.open_parallel(wl.num_branches)
    gb.open_parallel()
    chunk = np.full(wl.NB, 5, dtype=np.int32)
    compare(gb.parallel(chunk), tt.append_parallel(chunk), A.aspd_attn_branch_chunk, "chunk")
    ones = np.ones(wl.NB, dtype=np.int32)
    compare(gb.parallel(ones), tt.append_parallel(ones), A.aspd_attn_parallel_decode, "parallel")
    assert_state_equal(gb, tt)
    tt.merge()
    gb.merge()
    compare(gb.serial(one), tt.append_serial(one), A.aspd_attn_serial_decode, "serial after merge")
    assert_state_equal(gb, tt)


def test_two_calls_and_other_calls_share_a_workspace(A):
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5500, batch=2, prefix_range=(100, 400), branches_range=(2, 3), branch_len_range=(10, 50))
    layouts = W.random_layouts(wl, seed=2, fill=0.9)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts)
    _check_attention(A, gb, wl, step, tt, meta, label="first call")
    _check_attention(A, gb, wl, step, tt, meta, label="second call")
    # the same queries twice: a row group is computed whole by one workgroup in a fixed order, so which
    # workgroup took it does not show in the result
    q = wl.draw_q(meta.NQ).to(gb.dev)
    a = A.aspd_attn_full_sequence(gb.kv, gb.state, step, q, gb.workspace)
    b = A.aspd_attn_full_sequence(gb.kv, gb.state, step, q, gb.workspace)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    # and a call of another kind on the same workspace afterwards
    one = np.ones(wl.B, dtype=np.int32)
    m2 = tt.append_serial(one)
    s2 = gb.serial(one)
    q2 = wl.draw_q(m2.NQ)
    o2 = A.aspd_attn_serial_decode(gb.kv, gb.state, s2, q2.to(gb.dev), gb.workspace)
    torch.cuda.synchronize()
    ref, _ = attend(tt, m2, q2, wl.k_cache, wl.v_cache)
    assert np.abs(o2.float().cpu().numpy() - ref).max() <= TOL


def test_refused_layouts(A):
    """Branch runs not numbered 1..K, and a sequence that does not fit its block table: the sequence gets no
    tokens, the fault names the cause, the other sequences are served."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5600, batch=3, prefix_range=(40, 80), branches_range=(2, 3), branch_len_range=(5, 20))
    room = [16 * int((wl.block_tables[s] >= 0).sum()) for s in range(3)]
    good = [(0, 20), (1, 7), (2, 9), (0, 3)]
    for bad, bit in (([(0, 5), (2, 4)], 64), ([(1, 5), (3, 4)], 64), ([(0, 16 * wl.block_tables.shape[1] + 1)], 1)):
        layouts = [good, bad, good]
        gb = GpuBatch(wl)
        step = _build(A, gb, layouts)
        f = gb.fault()
        assert f & bit and f & A.FAULT_ROW_COUNT, (bad, f)
        assert gb.state.seq_len.cpu().numpy().tolist() == [39, 0, 39]
        # the two good sequences against the oracle: the refused one holds no tokens there either
        tt, meta = replay_layout(wl.block_tables, wl.block_size, [good, [], good])
        cu = step.cu_seq_new.cpu().numpy()
        nbad = sum(n for _, n in bad)
        assert cu.tolist() == [0, 39, 39 + nbad, 78 + nbad]
        q = wl.draw_q(int(cu[3]))
        out = torch.full((int(cu[3]), wl.num_q_heads, wl.head_dim), float("nan"), dtype=q.dtype, device=gb.dev)
        A.aspd_attn_full_sequence(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace, out=out)
        torch.cuda.synchronize()
        keep = np.r_[0:39, 39 + nbad:78 + nbad]
        ref, _ = attend(tt, meta, q[keep], wl.k_cache, wl.v_cache)
        got = out.float().cpu().numpy()
        assert np.abs(got[keep] - ref).max() <= TOL
        assert np.isnan(got[39:39 + nbad]).all()          # rows of the refused sequence: untouched
    assert room[0] >= 39


def test_argument_checks(A):
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5700, batch=2)
    gb = GpuBatch(wl)
    ones = np.ones(wl.B, dtype=np.int32)
    step = gb.serial(ones)                                # a step of the other metadata call
    q = wl.draw_q(step.NQ).to(gb.dev)
    with pytest.raises(A.AspdError) as e:
        A.aspd_attn_full_sequence(gb.kv, gb.state, step, q, gb.workspace)
    assert e.value.code == A.ERR_INVALID_ARG
    wf = W.random_small(seed=5701, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=2, batch=2)
    gf = GpuBatch(wf)
    assert A.aspd_sequence_plan_bytes(gf.kv, 2, 100) == 0
    with pytest.raises(A.AspdError) as e:
        _build(A, gf, [[(0, 5)], [(0, 6)]])
    assert e.value.code in (A.ERR_UNSUPPORTED, A.ERR_INVALID_ARG)


def test_edge_layouts(A):
    """A sequence without runs, one of empty runs only, a stage of one branch, a stage whose first branches are
    empty, two stages back to back, a sequence that starts and ends inside stages; grid capped to 3 workgroups."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5800, batch=6, num_q_heads=16, num_kv_heads=2, head_dim=64, prefix_range=(150, 200),
                        branches_range=(2, 3), branch_len_range=(20, 40))
    layouts = [[],
               [(0, 0), (1, 0), (2, 0), (0, 0)],
               [(0, 70), (1, 90), (0, 33)],
               [(0, 17), (1, 0), (2, 0), (3, 65), (0, 40)],
               [(0, 31), (1, 40), (2, 45), (1, 38), (2, 1), (3, 50), (0, 5)],
               [(1, 80), (2, 77), (0, 20), (1, 33), (2, 60)]]
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    cu, br, ln = _layout_arrays(layouts)
    step = A.aspd_build_sequence_meta(gb.kv, gb.state, gb._dev_i32(cu), gb._dev_i32(br), gb._dev_i32(ln), NQ=int(ln.sum()),
                                      max_workgroups=3)
    torch.cuda.synchronize()
    _check_meta(A, gb, wl, step, tt, meta, layouts)
    _check_attention(A, gb, wl, step, tt, meta, label="edge layouts, 3 workgroups")


def test_whole_sequence_call_in_a_hip_graph(A):
    """Metadata and attention of whole sequences captured in a HIP graph and replayed with eager launches on the same
    workspace in between: the work counter the launch takes its row groups from is back at zero after every launch,
    captured or not, and every replay gives the eager result bit for bit."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=5900, batch=3, prefix_range=(300, 700), branches_range=(2, 5), branch_len_range=(20, 80))
    layouts = W.random_layouts(wl, seed=4, fill=0.95)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    cu, br, ln = (gb._dev_i32(x) for x in _layout_arrays(layouts))
    step = A.aspd_build_sequence_meta(gb.kv, gb.state, cu, br, ln, NQ=meta.NQ)
    q = wl.draw_q(meta.NQ)
    qd = q.to(gb.dev)
    eager = A.aspd_attn_full_sequence(gb.kv, gb.state, step, qd, gb.workspace).clone()
    torch.cuda.synchronize()
    ref, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache)
    assert np.abs(eager.float().cpu().numpy() - ref).max() <= TOL
    out = torch.empty_like(qd)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        A.aspd_build_sequence_meta(gb.kv, gb.state, cu, br, ln, NQ=meta.NQ, step=step)   # warm-up on the side stream
        A.aspd_attn_full_sequence(gb.kv, gb.state, step, qd, gb.workspace, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        A.aspd_build_sequence_meta(gb.kv, gb.state, cu, br, ln, NQ=meta.NQ, step=step)
        A.aspd_attn_full_sequence(gb.kv, gb.state, step, qd, gb.workspace, out=out)
    for i in range(4):
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), i
        again = A.aspd_attn_full_sequence(gb.kv, gb.state, step, qd, gb.workspace)      # eager, same workspace
        torch.cuda.synchronize()
        assert torch.equal(again, eager), i
    assert gb.fault() == 0


def test_seeded_sweep_of_layouts(A):
    """Sixteen random batches (head layouts, head sizes, batch sizes, stage counts, position paradigms drawn per
    seed), metadata bit-exact and every row of the attention output against the oracle."""
    from gpu_drive import GpuBatch
    heads = [(32, 8, 128), (8, 8, 64), (16, 2, 128), (4, 1, 64), (12, 4, 128), (32, 4, 64)]
    for seed in range(16):
        rng = np.random.default_rng(9000 + seed)
        hq, hkv, d = heads[int(rng.integers(len(heads)))]
        wl = W.random_small(seed=6000 + seed, num_q_heads=hq, num_kv_heads=hkv, head_dim=d, batch=int(rng.integers(1, 7)),
                            prefix_range=(0, int(rng.integers(20, 500))), branches_range=(1, int(rng.integers(2, 9))),
                            branch_len_range=(1, int(rng.integers(5, 90))))
        layouts = W.random_layouts(wl, seed=seed, max_stages=int(rng.integers(1, 5)), max_branches=int(rng.integers(1, 12)),
                                   fill=float(rng.uniform(0.3, 1.0)))
        longest = max([n for r in layouts for b, n in r if b > 0] + [1])
        pm, pm_gpu = [("same_seq", A.POS_SAME_SEQ), ("same_max", A.POS_SAME_MAX),
                      (("fix", longest), A.POS_FIX_N(longest))][seed % 3]
        tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts, pm)
        gb = GpuBatch(wl)
        step = _build(A, gb, layouts, pos_mode=pm_gpu)
        _check_meta(A, gb, wl, step, tt, meta, layouts)
        if meta.NQ:
            _check_attention(A, gb, wl, step, tt, meta, label=f"sweep {seed}: {hq}/{hkv}/{d} B={wl.B} {pm}")


def test_shared_mask_is_plain_causal_attention(A):
    """shared_mask = 1: every row sees every slot up to its own, siblings included; against the oracle's shared
    mask and, for one head, against torch's causal attention."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=6100, batch=3, prefix_range=(100, 300), branches_range=(2, 5), branch_len_range=(10, 60))
    layouts = W.random_layouts(wl, seed=8, fill=0.9)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts)
    step.shared_mask = 1
    q = wl.draw_q(meta.NQ)
    out = A.aspd_attn_full_sequence(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace)
    torch.cuda.synchronize()
    ref, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache, shared_mask=True)
    got = out.float().cpu().numpy()
    assert np.abs(got - ref).max() <= TOL
    s, h = 1, 5
    r0, r1 = int(meta.cu_seq_new[s]), int(meta.cu_seq_new[s + 1])
    phys = torch.from_numpy(tt.physical_slots(s))
    k = wl.k_cache[phys // 16, h // 4, phys % 16].double()
    v = wl.v_cache[phys // 16, h // 4, phys % 16].double()
    sd = torch.nn.functional.scaled_dot_product_attention(q[r0:r1, h].double()[None], k[None], v[None], is_causal=True)[0]
    assert np.abs(got[r0:r1, h] - sd.numpy()).max() <= TOL
    # and the branch-isolating mask gives something else for the same rows
    step.shared_mask = 0
    iso = A.aspd_attn_full_sequence(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace).float().cpu().numpy()
    ref_iso, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache)
    assert np.abs(iso - ref_iso).max() <= TOL
    assert np.abs(iso - got).max() > 0.05


def test_re_prefill_with_rotary_append_end_to_end(A):
    """The three calls of a re-prefill in a row (Same-Re, Sec. 4.5.3): metadata of whole sequences, rotary encoding of
    all their tokens by the position ids of Eq. 4 with the K and V rows written into the cache, attention over the
    cache as written; against the oracle's chain of the same three steps in float64."""
    from gpu_drive import GpuBatch
    from oracle import rope_append
    wl = W.random_small(seed=6200, batch=3, num_q_heads=16, num_kv_heads=8, head_dim=128, prefix_range=(100, 500),
                        branches_range=(2, 5), branch_len_range=(10, 70))
    layouts = W.random_layouts(wl, seed=6, fill=0.9)
    tt, meta = replay_layout(wl.block_tables, wl.block_size, layouts)
    gb = GpuBatch(wl)
    step = _build(A, gb, layouts)
    NQ = meta.NQ
    g = torch.Generator().manual_seed(62)
    q = (torch.randn(NQ, wl.num_q_heads, wl.head_dim, generator=g) * wl.sigma).to(torch.bfloat16)
    k_new = (torch.randn(NQ, wl.num_kv_heads, wl.head_dim, generator=g) * wl.sigma).to(torch.bfloat16)
    v_new = (torch.randn(NQ, wl.num_kv_heads, wl.head_dim, generator=g) * wl.sigma).to(torch.bfloat16)
    k64 = gb.kv.k.double().cpu().numpy()
    v64 = gb.kv.v.double().cpu().numpy()
    q_dev = A.aspd_rope_append(gb.kv, step, q.to(gb.dev), k_new.to(gb.dev), v_new.to(gb.dev), 1e6)
    q_ref = rope_append(q.double().numpy(), k_new.double().numpy(), v_new.double().numpy(), meta.position_ids,
                        meta.slot_mapping, k64, v64, 1e6)
    out = A.aspd_attn_full_sequence(gb.kv, gb.state, step, q_dev, gb.workspace)
    torch.cuda.synchronize()
    assert np.abs(q_dev.double().cpu().numpy() - q_ref).max() <= TOL
    ref, _ = attend(tt, meta, torch.from_numpy(q_ref), torch.from_numpy(k64), torch.from_numpy(v64))
    err = np.abs(out.double().cpu().numpy() - ref).max()
    print(f"[re-prefill chain] rows={NQ} max|out-ref|={err:.3e}", flush=True)
    assert err <= TOL
