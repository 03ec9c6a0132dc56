"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Metadata and slot mapping must match bit-exactly; attention outputs within max-abs 1e-5 for fp32
inputs and 2e-2 for bf16 inputs (fp32 accumulation), the tolerances the benchmark spec states."""
import math

import numpy as np
import pytest
import torch

import aspd_workloads as W
from oracle import attend, TokenTable
from oracle_drive import table_with_prefix

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
LSE_TOL = {"f32": 2e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_08895_amd import binding
    binding.lib()  # fail loudly if the library is not built
    return binding


def _compare_attention(A, gb, tt, wl, step, meta, fn, rows=None, label="", check_step=True, shared_mask=False):
    from gpu_drive import assert_step_equal
    if check_step:
        assert_step_equal(step, meta)
    q = wl.draw_q(meta.NQ)
    lse = torch.full((meta.NQ, wl.num_q_heads), float("nan"), dtype=torch.float32, device=gb.dev)
    out = fn(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = attend(tt, meta, q, wl.k_cache, wl.v_cache, rows=rows, shared_mask=shared_mask)
    got = out.float().cpu().numpy().astype(np.float64)
    got_lse = lse.cpu().numpy().astype(np.float64)
    sel = np.arange(meta.NQ) if rows is None else np.asarray(rows)
    assert np.isfinite(got[sel]).all(), label
    err = np.abs(got[sel] - ref[sel]).max()
    lerr = np.abs(got_lse[sel] - ref_lse[sel]).max()
    print(f"[{label}] rows={sel.size} max|out-ref|={err:.3e} max|lse-ref|={lerr:.3e}", flush=True)
    assert err <= TOL[wl.dtype], (label, err)
    assert lerr <= LSE_TOL[wl.dtype], (label, lerr)
    return err


def _grow_both(A, wl, upto, check_every_step):
    """Oracle table and GPU batch after prefix + interleaved growth to `upto` tokens per branch."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    gb = GpuBatch(wl)
    tt = table_with_prefix(wl)
    step = gb.serial(wl.prefix_len)
    tt.open_parallel(wl.num_branches)
    gb.open_parallel()
    hist = W.interleaved_history(upto)
    for i, new_len in enumerate(hist):
        meta = tt.append_parallel(new_len)
        step = gb.parallel(new_len)
        if check_every_step or i >= len(hist) - 2:
            assert_step_equal(step, meta)
    assert_state_equal(gb, tt)
    return gb, tt


# --------------------------------------------------------------------------------------------- config 1
def test_config1_parallel_then_serial_fp32(A):
    from gpu_drive import assert_state_equal
    wl = W.config(1)
    gb, tt = _grow_both(A, wl, wl.branch_len - 1, True)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    assert meta.position_ids.tolist() == [68, 72, 79]
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label="cfg1 parallel")
    tt.merge()
    gb.merge()
    assert_state_equal(gb, tt)
    one = np.ones(wl.B, dtype=np.int32)
    meta = tt.append_serial(one)
    step = gb.serial(one)
    assert meta.position_ids.tolist() == [94] and meta.kv_len.tolist() == [95]
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label="cfg1 serial")
    assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- configs 2-4
@pytest.mark.parametrize("hinted", [False, True], ids=["no_hint", "hinted"])
@pytest.mark.parametrize("index", [2, 3, 4])
def test_config_parallel_decode_full_size(A, index, hinted):
    """`hinted`: with the bound on new tokens per sequence a decoding loop knows and bench.py passes
    (it selects the one- and two-tile kernels and their launch-to-launch records)."""
    wl = W.config(index)
    gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    if hinted:
        step.max_new_per_seq = int(wl.num_branches.max())
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label=f"cfg{index} parallel")
    if index == 4:
        # merge, then the 32 serial steps over prefix + all branches (all of them with the hints, the first
        # three without)
        from gpu_drive import assert_state_equal
        tt.merge()
        gb.merge()
        one = np.ones(wl.B, dtype=np.int32)
        for i in range(32 if hinted else 3):
            meta = tt.append_serial(one)
            step = gb.serial(one)
            if hinted:
                step.max_new_per_seq = 1
            _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label=f"cfg4 serial {i}")
        assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- config 5
@pytest.mark.parametrize("hinted", [False, True], ids=["no_hint", "hinted"])
@pytest.mark.parametrize("scale,batch", [(0.125, 8), (1.0, 64)])
def test_config5_chunk_then_decode(A, scale, batch, hinted):
    wl = W.config(5, scale=scale, batch=batch)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    chunk = np.full(wl.NB, 16, dtype=np.int32)
    meta = tt.append_parallel(chunk)
    step = gb.parallel(chunk)
    if hinted:
        step.max_new_per_seq = 16 * int(wl.num_branches.max())
    rows = None
    if scale == 1.0 and not hinted:   # full size without the hint: a seeded sample of the rows; with it: every row
        rows = np.sort(np.random.default_rng(5).choice(meta.NQ, size=256, replace=False))
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, rows=rows,
                       label=f"cfg5 chunk scale={scale}")
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    if hinted:
        step.max_new_per_seq = int(wl.num_branches.max())
    rows = None
    if scale == 1.0 and not hinted:
        rows = np.sort(np.random.default_rng(6).choice(meta.NQ, size=96, replace=False))
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, rows=rows,
                       label=f"cfg5 decode scale={scale}")


def test_chunk_launch_twice_gives_the_same_bits(A):
    """The row-splitting kernel fixes the order of every sum (each wave owns its rows, partial results are
    merged in the order of their key ranges), so two launches on the same inputs must agree bit for bit.
    A vector instruction that reads an MFMA result before the matrix unit has written it shows up here and,
    being within tolerance, nowhere else."""
    wl = W.config(5, scale=0.25, batch=16)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    chunk = np.full(wl.NB, 16, dtype=np.int32)
    meta = tt.append_parallel(chunk)
    step = gb.parallel(chunk)
    q = wl.draw_q(meta.NQ).to(gb.dev)
    outs = [A.aspd_attn_branch_chunk(gb.kv, gb.state, step, q, gb.workspace).clone() for _ in range(4)]
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o, outs[0])


LEAN = [dict(seed=901, head_dim=128, num_q_heads=32, num_kv_heads=8, prefix_range=(300, 900), chunk=16),
        dict(seed=902, head_dim=64, num_q_heads=8, num_kv_heads=2, prefix_range=(130, 700), chunk=24),
        dict(seed=903, head_dim=128, num_q_heads=4, num_kv_heads=4, prefix_range=(64, 400), chunk=40),
        dict(seed=904, head_dim=64, num_q_heads=16, num_kv_heads=1, prefix_range=(200, 600), chunk=7),
        dict(seed=905, head_dim=128, num_q_heads=8, num_kv_heads=1, prefix_range=(63, 65), chunk=33),
        dict(seed=906, head_dim=128, num_q_heads=32, num_kv_heads=8, prefix_range=(1000, 2200), chunk=3)]


@pytest.mark.parametrize("kw", LEAN, ids=lambda k: f"seed{k['seed']}")
def test_chunk_with_a_prefix_of_several_groups(A, kw):
    """Branch chunks behind prefixes of 4 to 140 pages, both head sizes, several row-group fillings (one wave to
    all eight, more than one row group): the leading page groups go through the row-splitting kernel's loop
    for fully visible groups, the branch region and the tail through the general one, and the boundary between
    the two falls at a different place for every wave."""
    kw = dict(kw)
    chunk_len = kw.pop("chunk")
    wl = W.random_small(batch=3, branches_range=(2, 6), branch_len_range=(1, 30), extra_tokens_per_branch=chunk_len + 4, **kw)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    chunk = np.full(wl.NB, chunk_len, dtype=np.int32)
    meta = tt.append_parallel(chunk)
    step = gb.parallel(chunk)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label=f"lean {kw['seed']}")
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label=f"lean {kw['seed']} decode")


# --------------------------------------------------------------------------------------------- mixed batches
@pytest.mark.parametrize("seed,dtype", [(21, "bf16"), (22, "f32")])
def test_mixed_batch_stages_switch_independently(A, seed, dtype):
    """Sequences open and end their parallel stages at different times; every call serves serial and
    parallel sequences together (MIXED append, per-sequence merge, branch renumbering).  Metadata
    bit-exact, attention against the dense-mask oracle, state equal after every call."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    rng = np.random.default_rng(seed)
    kw = dict(dtype=dtype, head_dim=64 if dtype == "f32" else 128, num_q_heads=4 if dtype == "f32" else 16,
              num_kv_heads=4, batch=6, prefix_range=(3, 90), branches_range=(4, 4), branch_len_range=(40, 40))
    wl = W.random_small(seed=seed, **kw)        # sizes the pools and block tables: <= 4 branches x 40 tokens
    gb = GpuBatch(wl)
    tt = table_with_prefix(wl)
    gb.serial(wl.prefix_len)
    B = wl.B
    K = [0] * B
    budget = [4 * 40 - 8] * B                   # tokens a sequence may still take
    for it in range(12):
        ending = [K[s] > 0 and rng.random() < 0.3 for s in range(B)]
        if any(ending):
            tt.merge(ending)
            gb.merge(ending)
            for s in range(B):
                if ending[s]:
                    K[s] = 0
        opening = [K[s] == 0 and rng.random() < 0.5 for s in range(B)]
        if any(ending) or any(opening):
            for s in range(B):
                if opening[s]:
                    K[s] = int(rng.integers(1, 5))
            tt.open_parallel(K)
            gb.renumber(K)
        chunky = it % 4 == 3
        nb, nm = [], []
        for s in range(B):
            if K[s]:
                n = rng.integers(0, 4 if chunky else 2, size=K[s])
                if n.sum() > budget[s]:
                    n[:] = 0
                nb.append(n)
                nm.append(0)
            else:
                nb.append(np.zeros(0, dtype=np.int64))
                nm.append(int(rng.integers(0, 3 if chunky else 2)) if budget[s] > 4 else 0)
            budget[s] -= int(nb[-1].sum()) + nm[-1]
        nbv = np.concatenate(nb)
        if nbv.sum() + sum(nm) == 0:
            continue
        meta = tt.append_mixed(nbv, nm)
        step = gb.mixed(nbv, nm)
        assert_step_equal(step, meta)
        fn = A.aspd_attn_branch_chunk if chunky else A.aspd_attn_parallel_decode
        _compare_attention(A, gb, tt, wl, step, meta, fn, label=f"mixed seed={seed} call {it}")
        assert_state_equal(gb, tt)


def test_mixed_rejects_main_tokens_under_open_branches(A):
    """A sequence with open branches cannot take a main-branch token: it is left as it was."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=31, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4, batch=2,
                        branches_range=(2, 2))
    gb = GpuBatch(wl)
    gb.serial(wl.prefix_len)
    gb.renumber([2, 0])
    before = gb.state.seq_len.cpu().numpy().copy()
    gb.mixed([1, 1], [1, 1])                     # sequence 0 owns branches and still asks for a main token
    after = gb.state.seq_len.cpu().numpy()
    assert gb.fault() & A.FAULT_STAGE
    assert after[0] == before[0] and after[1] == before[1] + 1


# --------------------------------------------------------------------------------------------- limits
def test_capped_grid_and_long_segments(A):
    """With the grid capped to two workgroups (aspd_step.max_workgroups) a 70 000-token sequence gives each
    of them more pages than the block-id window holds (512), so the kernels walk several windows; results
    must not depend on the cap.  The cap is set before the metadata call for the decode step (the step's
    plan is built for it) and after it for the chunk (the attention call then builds its own plan)."""
    wl = W.random_small(seed=61, dtype="bf16", head_dim=64, num_q_heads=2, num_kv_heads=1, batch=1,
                        prefix_range=(70000, 70000), branches_range=(3, 3), branch_len_range=(40, 40),
                        extra_tokens_per_branch=8)
    gb, tt = _grow_both(A, wl, np.minimum(wl.branch_len, 2) - 1, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_PARALLEL, gb._dev_i32(ones), NQ=int(ones.sum()),
                                    max_workgroups=2)
    assert step.plan_key != 0
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label="cap 2 parallel")
    chunk = np.full(wl.NB, 30, dtype=np.int32)           # 90 tokens x 2 heads: the row-splitting kernel
    meta = tt.append_parallel(chunk)
    step = gb.parallel(chunk)
    step.max_workgroups = 2
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label="cap 2 chunk")
    tt.merge()
    gb.merge()
    one = np.ones(wl.B, dtype=np.int32)
    meta = tt.append_serial(one)
    step = gb.serial(one)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label="uncapped serial")


@pytest.mark.parametrize("branches", [3, 6], ids=["one_tile", "two_tiles"])
def test_decode_loop_on_one_workspace(A, branches):
    """Forty consecutive decode launches on ONE workspace, with the hints a decoding loop gives (so the
    one- and two-tile kernels run, which start each launch from the record the last one left in the
    workspace): parallel steps, merge, serial steps, crossing page boundaries on the way.  Every third
    launch goes to a second cache that holds the same contents in other physical blocks, so a launch
    also meets a record whose segment is right and whose block ids are not."""
    import dataclasses
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    wl = W.random_small(seed=71, dtype="bf16", head_dim=128, num_q_heads=8, num_kv_heads=2, batch=2,
                        prefix_range=(6000, 9000), branches_range=(branches, branches), branch_len_range=(2, 2),
                        extra_tokens_per_branch=24, extra_tokens_per_seq=24)
    rng = np.random.default_rng(71)
    perm = rng.permutation(wl.num_blocks)
    order = torch.from_numpy(np.argsort(perm))
    bt = wl.block_tables
    wl2 = dataclasses.replace(wl, block_tables=np.where(bt >= 0, perm[np.maximum(bt, 0)], bt).astype(bt.dtype),
                              k_cache=wl.k_cache[order], v_cache=wl.v_cache[order])
    gbs = [GpuBatch(wl), GpuBatch(wl2)]
    gbs[1].workspace = gbs[0].workspace
    tt = table_with_prefix(wl)
    # a different batch of the same shape takes the same workspace now and then
    wl3 = W.random_small(seed=72, dtype="bf16", head_dim=128, num_q_heads=8, num_kv_heads=2, batch=2,
                         prefix_range=(6000, 9000), branches_range=(branches, branches), branch_len_range=(2, 2),
                         extra_tokens_per_branch=24, extra_tokens_per_seq=24)
    gb3, tt3 = _grow_both(A, wl3, wl3.branch_len, False)
    gb3.workspace = gbs[0].workspace
    for gb in gbs:
        gb.serial(wl.prefix_len)
        gb.open_parallel()
    tt.open_parallel(wl.num_branches)
    for new_len in W.interleaved_history(wl.branch_len):
        tt.append_parallel(new_len)
        for gb in gbs:
            gb.parallel(new_len)
    launch = 0

    def one(stage, new_len, hint, fn, label):
        nonlocal launch
        new_len = np.asarray(new_len, dtype=np.int32)
        meta = tt.append_parallel(new_len) if stage == A.STAGE_PARALLEL else tt.append_serial(new_len)
        steps = [A.aspd_build_branch_meta(gb.kv, gb.state, stage, gb._dev_i32(new_len), NQ=int(new_len.sum()),
                                          max_new_per_seq=hint) for gb in gbs]
        which = 1 if launch % 3 == 2 else 0
        # (the second cache's physical slots differ from the oracle's by construction)
        _compare_attention(A, gbs[which], tt, wl, steps[which], meta, fn, label=f"{label} {launch} cache {which}",
                           check_step=(which == 0))
        if launch % 5 == 4 and stage == A.STAGE_PARALLEL:
            meta3 = tt3.append_parallel(new_len)
            step3 = A.aspd_build_branch_meta(gb3.kv, gb3.state, stage, gb3._dev_i32(new_len), NQ=int(new_len.sum()),
                                             max_new_per_seq=hint)
            _compare_attention(A, gb3, tt3, wl3, step3, meta3, fn, label=f"{label} {launch} other batch")
        launch += 1

    for _ in range(20):
        one(A.STAGE_PARALLEL, np.ones(wl.NB), int(wl.num_branches.max()), A.aspd_attn_parallel_decode, "parallel")
    tt.merge()
    for gb in gbs:
        gb.merge()
    for _ in range(20):
        one(A.STAGE_SERIAL, np.ones(wl.B), 1, A.aspd_attn_serial_decode, "serial")
    assert_state_equal(gbs[0], tt)


def test_most_branches_one_sequence_can_have(A):
    """255 branches (owner tags are one byte): decode step and a 2-token chunk."""
    from gpu_drive import assert_state_equal
    wl = W.random_small(seed=62, dtype="bf16", head_dim=128, num_q_heads=8, num_kv_heads=2, batch=2,
                        prefix_range=(40, 300), branches_range=(255, 255), branch_len_range=(1, 4),
                        extra_tokens_per_branch=4)
    gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label="255 branches decode")
    two = np.full(wl.NB, 2, dtype=np.int32)
    meta = tt.append_parallel(two)
    step = gb.parallel(two)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label="255 branches chunk")
    assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- whole sequences
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_prefill_and_teacher_forced_branches(A, dtype):
    """Many tokens per call: a prompt prefilled through the serial call (causal among the new tokens, on
    top of tokens already cached), then every branch appended whole in one chunk call (the
    branch-sequential arrangement: a branch token sees the prefix and the earlier tokens of its own
    branch only), then a multi-token main-branch append after the merge."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    kw = dict(dtype=dtype, head_dim=64 if dtype == "f32" else 128, num_q_heads=4 if dtype == "f32" else 32,
              num_kv_heads=4 if dtype == "f32" else 8, batch=3, prefix_range=(200, 700), branches_range=(2, 5),
              branch_len_range=(30, 150), extra_tokens_per_seq=80)
    wl = W.random_small(seed=51, **kw)
    gb = GpuBatch(wl)
    tt = TokenTable(wl.block_tables, wl.block_size)

    def serial(new_len, label):
        new_len = np.asarray(new_len, dtype=np.int32)
        meta = tt.append_serial(new_len)
        step = A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_SERIAL, gb._dev_i32(new_len), NQ=int(new_len.sum()),
                                        max_new_per_seq=int(new_len.max()))
        assert_step_equal(step, meta)
        _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label=label)

    first = wl.prefix_len // 3
    serial(first, "prefill part 1")
    serial(wl.prefix_len - first, "prefill part 2")
    tt.open_parallel(wl.num_branches)
    gb.open_parallel()
    meta = tt.append_parallel(wl.branch_len)          # every branch whole, one call
    step = gb.parallel(wl.branch_len)
    assert_step_equal(step, meta)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label="teacher-forced branches")
    tt.merge()
    gb.merge()
    serial(np.full(wl.B, 40), "main branch after merge, 40 tokens")
    assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- rotary append
@pytest.mark.parametrize("seed,dtype,theta", [(41, "f32", 10000.0), (42, "bf16", 1e6), (43, "bf16", 10000.0)])
def test_rope_append_then_attention(A, seed, dtype, theta):
    """Metadata -> rotary encoding + cache append -> attention, against the oracle's chain of the same
    three steps.  Checked: the rotated queries, every cache row written, that nothing else in the
    pools changed, and the attention outputs computed from the cache the kernel wrote."""
    from oracle import rope_append
    kw = dict(dtype=dtype, head_dim=64 if dtype == "f32" else 128, num_q_heads=4 if dtype == "f32" else 16,
              num_kv_heads=4 if dtype == "f32" else 8, batch=4, prefix_range=(20, 3000))
    wl = W.random_small(seed=seed, **kw)
    gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
    tol = TOL[wl.dtype]
    rng = np.random.default_rng(seed)
    for new_len, fn in ((np.ones(wl.NB, dtype=np.int32), A.aspd_attn_parallel_decode),
                        (rng.integers(0, 4, size=wl.NB).astype(np.int32), A.aspd_attn_branch_chunk)):
        meta = tt.append_parallel(new_len)
        step = gb.parallel(new_len)
        NQ = meta.NQ
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        g = torch.Generator().manual_seed(seed + NQ)
        q = (torch.randn(NQ, wl.num_q_heads, wl.head_dim, generator=g) * wl.sigma).to(tdt)
        k_new = (torch.randn(NQ, wl.num_kv_heads, wl.head_dim, generator=g) * wl.sigma).to(tdt)
        v_new = (torch.randn(NQ, wl.num_kv_heads, wl.head_dim, generator=g) * wl.sigma).to(tdt)
        k_before, v_before = gb.kv.k.clone(), gb.kv.v.clone()
        q_dev = A.aspd_rope_append(gb.kv, step, q.to(gb.dev), k_new.to(gb.dev), v_new.to(gb.dev), theta)
        torch.cuda.synchronize()
        # oracle chain, float64 throughout, on copies of the pools as they were before the call
        k64 = k_before.double().cpu().numpy()
        v64 = v_before.double().cpu().numpy()
        q_ref = rope_append(q.double().numpy(), k_new.double().numpy(), v_new.double().numpy(), meta.position_ids,
                            meta.slot_mapping, k64, v64, theta)
        assert np.abs(q_dev.double().cpu().numpy() - q_ref).max() <= tol
        k_got, v_got = gb.kv.k.double().cpu().numpy(), gb.kv.v.double().cpu().numpy()
        written = np.zeros(k64.shape[0] * 16, dtype=bool)
        written[meta.slot_mapping] = True
        written = written.reshape(-1, 16)
        kt, vt = k_got.transpose(0, 2, 1, 3), v_got.transpose(0, 2, 1, 3)      # [blocks][16][Hkv][D]
        kr, vr = k64.transpose(0, 2, 1, 3), v64.transpose(0, 2, 1, 3)
        assert np.abs(kt[written] - kr[written]).max() <= tol
        assert np.array_equal(vt[written], vr[written])                        # values are copied, not computed
        same = lambda a, b: np.array_equal(a, b, equal_nan=True)               # unmapped blocks hold NaN
        assert same(kt[~written], kr[~written]) and same(vt[~written], vr[~written])
        # attention on the cache the kernel wrote, against the oracle on the cache the oracle wrote
        lse = torch.full((NQ, wl.num_q_heads), float("nan"), dtype=torch.float32, device=gb.dev)
        out = fn(gb.kv, gb.state, step, q_dev, gb.workspace, lse=lse)
        torch.cuda.synchronize()
        ref, _ = attend(tt, meta, torch.from_numpy(q_ref), torch.from_numpy(k64), torch.from_numpy(v64))
        err = np.abs(out.double().cpu().numpy() - ref).max()
        print(f"[rope seed={seed} {fn.__name__}] rows={NQ} max|out-ref|={err:.3e}", flush=True)
        assert err <= tol


# --------------------------------------------------------------------------------------------- position paradigms
@pytest.mark.parametrize("mode", ["same_max", ("fix", 48)])
def test_position_paradigms_of_the_ablation(A, mode):
    """Same-Max and fixed-interval position ids (Sec. 4.5.3) through all metadata stages, over two
    rounds of parallel decoding with sequences switching independently: position ids and every other
    output bit-exact against the oracle run in the same paradigm; attention is the same as ever."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    seed = 71
    rng = np.random.default_rng(seed)
    wl = W.random_small(seed=seed, dtype="bf16", head_dim=128, num_q_heads=8, num_kv_heads=4, batch=5,
                        prefix_range=(5, 120), branches_range=(4, 4), branch_len_range=(40, 40))
    gb = GpuBatch(wl)
    gb.state.pos_mode = A.POS_SAME_MAX if mode == "same_max" else A.POS_FIX_N(mode[1])
    tt = TokenTable(wl.block_tables, wl.block_size, pos_mode=mode)
    meta = tt.append_serial(wl.prefix_len)
    step = gb.serial(wl.prefix_len)
    assert_step_equal(step, meta)
    B = wl.B
    K = [0] * B
    held = [0] * B                                # tokens in the longest branch of the running stage
    budget = [4 * 40 - 8] * B
    for it in range(14):
        ending = [K[s] > 0 and rng.random() < 0.3 for s in range(B)]   # also stages that hold no token yet
        if any(ending):
            tt.merge(ending)
            gb.merge(ending)
            for s in range(B):
                if ending[s]:
                    K[s], held[s] = 0, 0
        opening = [K[s] == 0 and rng.random() < 0.5 for s in range(B)]
        if any(ending) or any(opening):
            for s in range(B):
                if opening[s]:
                    K[s] = int(rng.integers(1, 5))
            tt.open_parallel(K)
            gb.renumber(K)
        nb, nm = [], []
        for s in range(B):
            if K[s]:
                n = rng.integers(0, 4, size=K[s])
                if n.sum() > budget[s] or held[s] + 3 > 40:
                    n[:] = 0
                nb.append(n)
                nm.append(0)
                held[s] += int(n.max()) if n.size else 0
            else:
                nb.append(np.zeros(0, dtype=np.int64))
                nm.append(int(rng.integers(0, 3)) if budget[s] > 4 else 0)
            budget[s] -= int(nb[-1].sum()) + nm[-1]
        nbv = np.concatenate(nb)
        if nbv.sum() + sum(nm) == 0:
            continue
        meta = tt.append_mixed(nbv, nm)
        step = gb.mixed(nbv, nm)
        assert_step_equal(step, meta)
        _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label=f"{mode} call {it}")
        assert_state_equal(gb, tt)
        assert np.array_equal(gb.state.main_pos.cpu().numpy(), np.array(tt.next_main_pos, dtype=np.int32))
    assert gb.fault() == 0


@pytest.mark.parametrize("mode,want", [("same_seq", [0, 1, 2, 3, 3]), ("same_max", [0, 1, 2, 3, 3]),
                                       (("fix", 4), [0, 1, 10, 11, 15])])
def test_stage_that_ends_without_a_token(A, mode, want):
    """The hand-derived lines "empty ..." of tests/golden/position_paradigms.txt, replayed on the GPU: a
    stage is opened and merged before any branch produced a token; fixed intervals stay spent
    (Sec. 4.5.3, "pre-allocated"), the other paradigms continue where the main branch stood."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    wl = W.random_small(seed=73, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4, batch=1,
                        prefix_range=(2, 2), branches_range=(2, 2), branch_len_range=(4, 4))
    gb = GpuBatch(wl)
    gb.state.pos_mode = {"same_seq": A.POS_SAME_SEQ, "same_max": A.POS_SAME_MAX}.get(mode) if isinstance(mode, str) \
        else A.POS_FIX_N(mode[1])
    tt = TokenTable(wl.block_tables, wl.block_size, pos_mode=mode)
    got = []
    for op, arg in (("serial", [2]), ("open", [2]), ("merge", None), ("serial", [1]), ("open", [2]), ("step", [1, 1])):
        if op == "serial":
            meta, step = tt.append_serial(arg), gb.serial(arg)
        elif op == "open":
            tt.open_parallel(arg)
            gb.renumber(arg)
            continue
        elif op == "merge":
            tt.merge()
            gb.merge()
            assert_state_equal(gb, tt)
            continue
        else:
            meta, step = tt.append_parallel(arg), gb.parallel(arg)
        assert_step_equal(step, meta)
        got += step.position_ids.cpu().numpy()[:meta.NQ].tolist()
    assert got == want
    assert_state_equal(gb, tt)
    assert np.array_equal(gb.state.main_pos.cpu().numpy(), np.array(tt.next_main_pos, dtype=np.int32))


def test_serial_rejects_main_tokens_under_an_unmerged_stage(A):
    """Main-branch tokens through the SERIAL stage for a sequence whose branches hold tokens that have not
    been merged: the sequence is left as it was (its position would fall into the branches' range)."""
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=32, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4, batch=2,
                        branches_range=(2, 2))
    gb = GpuBatch(wl)
    gb.serial(wl.prefix_len)
    gb.renumber([2, 0])
    gb.mixed([1, 1], [0, 0])
    assert gb.fault() == 0
    before = gb.state.seq_len.cpu().numpy().copy()
    base = gb.state.stage_base.cpu().numpy().copy()
    gb.serial(np.array([1, 1], dtype=np.int32))   # sequence 0 is still in its parallel stage
    after = gb.state.seq_len.cpu().numpy()
    assert gb.fault() & A.FAULT_STAGE
    assert after[0] == before[0] and after[1] == before[1] + 1
    assert gb.state.stage_base.cpu().numpy()[0] == base[0]


def test_fixed_interval_overflow_is_refused(A):
    from gpu_drive import GpuBatch
    wl = W.random_small(seed=72, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4, batch=1,
                        branches_range=(2, 2), branch_len_range=(20, 20))
    gb = GpuBatch(wl)
    gb.state.pos_mode = A.POS_FIX_N(4)
    gb.serial(wl.prefix_len)
    gb.renumber([2])
    gb.parallel(np.array([3, 4], dtype=np.int32))
    assert gb.fault() == 0
    before = gb.state.seq_len.cpu().numpy().copy()
    gb.parallel(np.array([2, 0], dtype=np.int32))          # branch 0 would hold 5 > 4 positions
    assert gb.fault() & A.FAULT_INTERVAL
    assert np.array_equal(gb.state.seq_len.cpu().numpy(), before)


# --------------------------------------------------------------------------------------------- many sequences
def test_large_batch_decode_and_serial(A):
    """More sequences than a wave has lanes (the schedule's search over sequences takes its other path)
    and more units than workgroups: config 3's mix, 150 sequences, short prefixes."""
    from gpu_drive import assert_state_equal
    wl = W.config(3, scale=0.06, batch=150)
    gb, tt = _grow_both(A, wl, np.minimum(wl.branch_len, 24) - 1, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label="batch150 parallel")
    chunk = np.full(wl.NB, 3, dtype=np.int32)
    meta = tt.append_parallel(chunk)
    step = gb.parallel(chunk)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label="batch150 chunk")
    tt.merge()
    gb.merge()
    one = np.ones(wl.B, dtype=np.int32)
    meta = tt.append_serial(one)
    step = gb.serial(one)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label="batch150 serial")
    assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- randomized small
SMALL = [
    dict(seed=101, dtype="bf16", head_dim=128, num_q_heads=32, num_kv_heads=8),
    dict(seed=102, dtype="bf16", head_dim=128, num_q_heads=8, num_kv_heads=8, branches_range=(1, 12)),
    dict(seed=103, dtype="bf16", head_dim=64, num_q_heads=16, num_kv_heads=4),
    dict(seed=104, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4),
    dict(seed=105, dtype="f32", head_dim=128, num_q_heads=8, num_kv_heads=2),
    dict(seed=106, dtype="bf16", head_dim=128, num_q_heads=32, num_kv_heads=8, prefix_range=(0, 0)),
    dict(seed=107, dtype="bf16", head_dim=128, num_q_heads=32, num_kv_heads=8, branches_range=(9, 14),
         prefix_range=(100, 300)),
    dict(seed=108, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=1, branches_range=(1, 3)),
]


@pytest.mark.parametrize("kw", SMALL, ids=lambda k: f"seed{k['seed']}")
def test_random_small_all_calls(A, kw):
    from gpu_drive import assert_state_equal
    wl = W.random_small(**kw)
    gb, tt = _grow_both(A, wl, wl.branch_len, True)
    rng = np.random.default_rng(kw["seed"])
    # a ragged chunk, some branches getting nothing
    chunk = rng.integers(0, 7, size=wl.NB).astype(np.int32)
    if chunk.sum() == 0:
        chunk[0] = 3
    meta = tt.append_parallel(chunk)
    step = gb.parallel(chunk)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_branch_chunk, label=f"{wl.name} chunk")
    # a decode step in which some branches have finished
    active = (rng.random(wl.NB) < 0.7).astype(np.int32)
    if active.sum() == 0:
        active[-1] = 1
    meta = tt.append_parallel(active)
    step = gb.parallel(active)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label=f"{wl.name} decode")
    assert_state_equal(gb, tt)
    # merge and two serial steps
    tt.merge()
    gb.merge()
    for i in range(2):
        one = np.ones(wl.B, dtype=np.int32)
        meta = tt.append_serial(one)
        step = gb.serial(one)
        _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label=f"{wl.name} serial {i}")
    assert_state_equal(gb, tt)


def test_second_parallel_round_sees_first_rounds_branches(A):
    """Iterative serial-parallel switching (Sec. 3.3): a later stage attends earlier branches."""
    from gpu_drive import assert_state_equal
    wl = W.random_small(120, batch=2, extra_tokens_per_branch=30, extra_tokens_per_seq=40)
    gb, tt = _grow_both(A, wl, wl.branch_len, True)
    tt.merge()
    gb.merge()
    two = np.full(wl.B, 2, dtype=np.int32)
    meta = tt.append_serial(two)     # two main tokens at once: the second must not see... it sees the first
    step = gb.serial(two)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label="round2 serial x2")
    tt.open_parallel(wl.num_branches)
    gb.open_parallel()
    for i in range(3):
        ones = np.ones(wl.NB, dtype=np.int32)
        meta = tt.append_parallel(ones)
        step = gb.parallel(ones)
        _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label=f"round2 step {i}")
    assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- invariants on the GPU
def test_sibling_kv_does_not_reach_a_branch(A):
    """Perturbing the K/V of sibling branches (to huge finite values) must not change any output:
    masked weights are exactly zero, Sec. 3.2 "mutual invisibility across branches".  The bf16 kernel
    hands page pairs to waves dynamically, so two runs may sum in a different order: outputs are
    compared to a few bf16 ulps, while a leak of a sibling key would show up at the 1e30 scale."""
    wl = W.random_small(130, batch=2, branches_range=(3, 5), branch_len_range=(5, 30))
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    q = wl.draw_q(meta.NQ).to(gb.dev)
    base = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace).clone()
    cu = wl.cu_branches
    for r in range(meta.NQ):
        s = int(meta.q_seq[r])
        tag = int(meta.q_branch[r]) - int(cu[s]) + 1
        k2, v2 = gb.kv.k.clone(), gb.kv.v.clone()
        for j in range(int(wl.prefix_len[s]), len(tt.pos[s])):
            if tt.branch[s][j] != tag:
                ph = tt.physical_slot(s, j)
                k2[ph // 16, :, ph % 16] = 1e30 if j % 2 else -3e4
                v2[ph // 16, :, ph % 16] = -1e30
        kv2 = A.KVCache(k2, v2, gb.kv.block_tables, gb.kv.num_q_heads)
        out = A.aspd_attn_parallel_decode(kv2, gb.state, step, q, gb.workspace)
        assert torch.isfinite(out[r].float()).all(), r
        assert (out[r].float() - base[r].float()).abs().max().item() <= 4e-3, r


def test_permuting_the_branches_permutes_the_outputs(A):
    """Eq. 3 knows no order among the branches of a stage: the same branches (their K/V rows and queries)
    laid into the cache in another branch order give every branch the output it had, to rounding (the keys
    of a row are then summed in another order).  Decode step and a 3-token chunk."""
    import dataclasses
    from gpu_drive import GpuBatch
    from oracle_drive import table_at
    wl = W.random_small(134, batch=3, prefix_range=(30, 400), branches_range=(3, 6), branch_len_range=(4, 30),
                        extra_tokens_per_branch=8)
    rng = np.random.default_rng(134)
    cu = wl.cu_branches
    # branch k of the permuted layout is branch perm[k] of the original one, per sequence
    perm = np.concatenate([cu[s] + rng.permutation(int(wl.num_branches[s])) for s in range(wl.B)])
    for new_tokens, fn in ((1, "aspd_attn_parallel_decode"), (3, "aspd_attn_branch_chunk")):
        new_len = np.full(wl.NB, new_tokens, dtype=np.int32)
        # the two layouts as the oracle's tables have them: (sequence, branch, index in branch) -> slot
        wl_p = dataclasses.replace(wl, branch_len=wl.branch_len[perm].copy())
        tabs, metas = [], []
        for w in (wl, wl_p):
            tt = table_at(w, w.branch_len)
            metas.append(tt.append_parallel(new_len))
            tabs.append(tt)

        def where(tt, s):   # (branch number 1.., index in branch) -> physical slot, for the running stage
            return {(tt.branch[s][j], tt.index_in_branch[s][j]): tt.physical_slot(s, j)
                    for j in range(int(wl.prefix_len[s]), len(tt.pos[s]))}
        k_p, v_p = wl.k_cache.clone(), wl.v_cache.clone()
        for s in range(wl.B):
            a, b = where(tabs[0], s), where(tabs[1], s)
            K = int(wl.num_branches[s])
            for kb in range(K):
                ka = int(perm[cu[s] + kb] - cu[s])           # original number of the permuted layout's branch kb
                for t in range(int(wl_p.branch_len[cu[s] + kb]) + new_tokens):
                    src, dst = a[(ka + 1, t)], b[(kb + 1, t)]
                    k_p[dst // 16, :, dst % 16] = wl.k_cache[src // 16, :, src % 16]
                    v_p[dst // 16, :, dst % 16] = wl.v_cache[src // 16, :, src % 16]
        wl_p = dataclasses.replace(wl_p, k_cache=k_p, v_cache=v_p)
        # rows: packed by (sequence, branch, token); row of (branch kb, token j) in the permuted call is the row
        # of (branch perm[kb], token j) in the original call
        q = wl.draw_q(metas[0].NQ)
        row_p = np.concatenate([np.arange(new_tokens) + new_tokens * perm[g] for g in range(wl.NB)])
        outs = []
        for w, qq in ((wl, q), (wl_p, q[row_p])):
            gb = GpuBatch(w)
            gb.grow_to(w.branch_len)
            step = gb.parallel(new_len)
            outs.append(getattr(A, fn)(gb.kv, gb.state, step, qq.to(gb.dev), gb.workspace).float().cpu())
            assert gb.fault() == 0
        assert torch.isfinite(outs[0]).all()
        assert (outs[1] - outs[0][row_p]).abs().max().item() <= 4e-3, fn


def test_unwritten_slots_may_hold_anything(A):
    """The slots of a sequence's last page past its last token have never been written and blocks the
    tables do not use belong to somebody else: both are filled with NaN here, K and V alike.  No call may
    let them reach an output (a masked key has weight zero, and zero times NaN is NaN)."""
    from gpu_drive import GpuBatch, assert_state_equal
    for kw in (dict(), dict(dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=2)):
        wl = W.random_small(135, batch=4, prefix_range=(5, 300), branches_range=(2, 5), **kw)
        gb, tt = _grow_both(A, wl, wl.branch_len, False)

        def poison():
            k, v = gb.kv.k, gb.kv.v
            for s in range(wl.B):
                T = len(tt.pos[s])
                cap = int((wl.block_tables[s] >= 0).sum()) * 16
                for j in range(T, cap):
                    ph = int(wl.block_tables[s, j // 16]) * 16 + j % 16
                    k[ph // 16, :, ph % 16] = float("nan")
                    v[ph // 16, :, ph % 16] = float("nan")

        def write_rows(meta):   # the new tokens' K/V: finite values where the step put them
            g = torch.Generator().manual_seed(int(meta.NQ))
            for ph in meta.slot_mapping.tolist():
                for cache, host in ((gb.kv.k, wl.k_cache), (gb.kv.v, wl.v_cache)):
                    row = (torch.randn(wl.num_kv_heads, wl.head_dim, generator=g) * wl.sigma).to(wl.torch_dtype)
                    cache[ph // 16, :, ph % 16] = row.to(gb.dev)
                    host[ph // 16, :, ph % 16] = row

        poison()
        for new_len, fn in ((np.ones(wl.NB, dtype=np.int32), A.aspd_attn_parallel_decode),
                            (np.full(wl.NB, 3, dtype=np.int32), A.aspd_attn_branch_chunk)):
            meta = tt.append_parallel(new_len)
            step = gb.parallel(new_len)
            write_rows(meta)
            _compare_attention(A, gb, tt, wl, step, meta, fn, label=f"poisoned {fn.__name__} {wl.dtype}")
        tt.merge()
        gb.merge()
        one = np.ones(wl.B, dtype=np.int32)
        meta = tt.append_serial(one)
        step = gb.serial(one)
        write_rows(meta)
        _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_serial_decode, label=f"poisoned serial {wl.dtype}")
        assert_state_equal(gb, tt)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_shared_mask_of_the_ablation(A, dtype):
    """aspd_step.shared_mask: branch rows attend like main-branch rows (every slot up to their own, siblings
    included), set before the metadata call (the step's plan is built for it) and after it (the attention
    call builds its own); decode step and chunk."""
    from gpu_drive import GpuBatch
    kw = dict(dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=2) if dtype == "f32" else {}
    wl = W.random_small(136, batch=3, prefix_range=(20, 500), branches_range=(2, 6), **kw)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    for new_tokens, fn, before in ((1, A.aspd_attn_parallel_decode, True), (4, A.aspd_attn_branch_chunk, False)):
        new_len = np.full(wl.NB, new_tokens, dtype=np.int32)
        meta = tt.append_parallel(new_len)
        step = A.Step(int(new_len.sum()), wl.NB, wl.B, gb.dev, max_new_per_seq=new_tokens * int(wl.num_branches.max()))
        step.shared_mask = 1 if before else 0
        A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_PARALLEL, gb._dev_i32(new_len), step=step)
        step.shared_mask = 1
        err_shared = _compare_attention(A, gb, tt, wl, step, meta, fn, label=f"shared mask {fn.__name__}", shared_mask=True)
        # and the flag does change what is computed: the same call without it matches the independent mask
        step.shared_mask = 0
        _compare_attention(A, gb, tt, wl, step, meta, fn, label=f"independent mask {fn.__name__}")
        assert err_shared <= TOL[wl.dtype]


def test_engine_drives_the_library_like_the_oracle(A):
    """The host engine (special-token state machine, Sec. 3.3) on the HIP library, in lockstep with the same
    engine logic on the oracle's token table: every step's metadata bit-exact, every step's attention (the
    entry point the engine names) against the dense-mask oracle on K/V rows written at the step's slots."""
    from engine_drive import OracleDriver, ScriptedModel
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    from paper_2508_08895_amd.engine import HybridEngine, LibraryDriver, SpecialTokens
    SP = SpecialTokens(901, 902, 903, 904, 905, 906, 999, prefix_sep=(907,))
    wl = W.random_small(137, batch=3, prefix_range=(5, 5), branches_range=(3, 3), branch_len_range=(40, 40),
                        extra_tokens_per_seq=60)                  # sizes pools and tables only
    gb = GpuBatch(wl)
    lib, orc = LibraryDriver(A, gb.kv, gb.state), OracleDriver(wl.block_tables, wl.block_size)

    class Tee:
        def serial(self, n, hint):
            self.meta = orc.serial(n, hint)
            return lib.serial(n, hint)

        def mixed(self, nb, nm, hint):
            self.meta = orc.mixed(nb, nm, hint)
            return lib.mixed(nb, nm, hint)

        def renumber(self, k):
            orc.renumber(k)
            lib.renumber(k)

        def merge(self, which):
            orc.merge(which)
            lib.merge(which)

    tee = Tee()
    eng = HybridEngine(tee, SP, batch=wl.B)

    def titles(*ts):
        out = []
        for t in ts:
            out += [SP.title_open, *t, SP.title_close]
        return out + [SP.para_open]

    main = [[40, 41, 42, 43, 44, 45, SP.eos],
            [*titles([11, 12], [21]), 51, *titles([31], [11, 12]), 52, SP.eos],
            [60, 61, *titles([11], [21, 22], [31]), 63, SP.eos]]
    stages = [[],
              [[[1, 2, 3, SP.branch_close], [4, SP.branch_close]], [[5, SP.branch_close], [6, 7, SP.branch_close]]],
              [[[8, SP.branch_close], [9, 9, 9, 9, SP.branch_close], [SP.branch_close]]]]
    model = ScriptedModel(main, stages)
    g = torch.Generator().manual_seed(137)
    plan = eng.prefill([[1], [2, 2], [3, 3, 3]])
    steps = 0
    while plan is not None:
        meta = tee.meta
        assert_step_equal(plan.step, meta)
        # the new tokens' K/V rows, where the step says they go (device cache and the oracle's host copy)
        for ph in meta.slot_mapping.tolist():
            for cache, host in ((gb.kv.k, wl.k_cache), (gb.kv.v, wl.v_cache)):
                row = (torch.randn(wl.num_kv_heads, wl.head_dim, generator=g) * wl.sigma).to(wl.torch_dtype)
                cache[ph // 16, :, ph % 16] = row.to(gb.dev)
                host[ph // 16, :, ph % 16] = row
        _compare_attention(A, gb, orc.tt, wl, plan.step, meta, getattr(A, plan.attention), label=f"engine step {steps} {plan.attention}",
                           check_step=False)
        eng.accept(model(eng, plan))
        assert_state_equal(gb, orc.tt)
        plan = eng.next_step()
        steps += 1
    assert eng.finished() and [s.stages for s in eng.seqs] == [0, 2, 1]
    # Re-prefill (the Same-Re reading of Sec. 4.5.3): the sequences the engine produced, laid out whole in the
    # training arrangement and rebuilt from slot 0 in one metadata call and one attention launch; against the
    # oracle's replay of the same layouts.
    from oracle.sequence_layout import replay_layout
    layouts = [eng.layout(s)[0] for s in range(wl.B)]
    t2, meta2 = replay_layout(wl.block_tables, wl.block_size, layouts)
    step2 = lib.reprefill(layouts)
    torch.cuda.synchronize()
    for f in ("cu_seq_new", "q_seq", "position_ids", "logical_slot", "slot_mapping", "kv_len"):
        got = getattr(step2, f).cpu().numpy()
        assert np.array_equal(got if f == "cu_seq_new" else got[:meta2.NQ], getattr(meta2, f)), f
    _compare_attention(A, gb, t2, wl, step2, meta2, A.aspd_attn_full_sequence, label="engine re-prefill", check_step=False)


def test_repeat_calls_agree(A):
    """Two runs of the same call agree to rounding (see the note on summation order above)."""
    wl = W.random_small(131, batch=4)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    step = gb.parallel(ones)
    q = wl.draw_q(step.NQ).to(gb.dev)
    a = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace).clone()
    b = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace)
    assert (a.float() - b.float()).abs().max().item() <= 4e-3


def test_a_captured_step_replays_like_the_eager_one(A):
    """No call reads device data on the host, so a whole decode step (state restored from a snapshot,
    metadata, attention; then merge, metadata and attention of a serial step) can be captured in a HIP
    graph.  Five replays, with eager launches on the same workspace and synchronisations between them,
    each leave the step arrays, the state and the outputs the eager step left, and the oracle's."""
    from gpu_drive import assert_step_equal, assert_state_equal
    wl = W.config(3, scale=0.12, batch=6)
    gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
    st = gb.state
    live = [st.stage_base, st.seq_len, st.branch_len, st.slot_owner, st.main_pos]
    snap = [t.clone() for t in live]
    ones = np.ones(wl.NB, dtype=np.int32)
    one = np.ones(wl.B, dtype=np.int32)
    d_ones, d_one = gb._dev_i32(ones), gb._dev_i32(one)
    # eager step, checked against the oracle
    meta_p = tt.append_parallel(ones)
    step_p = gb.parallel(ones)
    assert_step_equal(step_p, meta_p)
    q_p = wl.draw_q(meta_p.NQ)
    ref_p, _ = attend(tt, meta_p, q_p, wl.k_cache, wl.v_cache)
    q_p = q_p.to(gb.dev)
    eager_p = A.aspd_attn_parallel_decode(gb.kv, st, step_p, q_p, gb.workspace).clone()
    tt.merge()
    gb.merge()
    meta_s = tt.append_serial(one)
    step_s = gb.serial(one)
    assert_step_equal(step_s, meta_s)
    q_s = wl.draw_q(meta_s.NQ)
    ref_s, _ = attend(tt, meta_s, q_s, wl.k_cache, wl.v_cache)
    q_s = q_s.to(gb.dev)
    eager_s = A.aspd_attn_serial_decode(gb.kv, st, step_s, q_s, gb.workspace).clone()
    torch.cuda.synchronize()
    assert np.abs(eager_p.float().cpu().numpy() - ref_p).max() <= TOL[wl.dtype]
    assert np.abs(eager_s.float().cpu().numpy() - ref_s).max() <= TOL[wl.dtype]
    assert_state_equal(gb, tt)
    end_state = [t.clone() for t in live]
    out_p, out_s = torch.empty_like(eager_p), torch.empty_like(eager_s)

    def one_step():
        for dst, src in zip(live, snap):
            dst.copy_(src)
        A.aspd_build_branch_meta(gb.kv, st, A.STAGE_PARALLEL, d_ones, step=step_p)
        A.aspd_attn_parallel_decode(gb.kv, st, step_p, q_p, gb.workspace, out=out_p)
        A.aspd_build_branch_meta(gb.kv, st, A.STAGE_MERGE, None)
        A.aspd_build_branch_meta(gb.kv, st, A.STAGE_SERIAL, d_one, step=step_s)
        A.aspd_attn_serial_decode(gb.kv, st, step_s, q_s, gb.workspace, out=out_s)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_step()
    for i in range(5):
        # eager work between the replays: scribble over what the graph has to produce, and use the
        # workspace for another launch (a chunk call, another kernel) so that the replay meets its records
        out_p.fill_(float("nan"))
        out_s.fill_(float("nan"))
        for t in (step_p.position_ids, step_p.logical_slot, step_s.position_ids, step_s.slot_mapping):
            t.fill_(-7)
        A.aspd_attn_branch_chunk(gb.kv, st, step_s, q_s, gb.workspace)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_step_equal(step_p, meta_p)
        assert_step_equal(step_s, meta_s)
        for t, e in zip(live, end_state):
            assert torch.equal(t, e), i
        # (pairs of pages are handed to waves dynamically: two runs agree to rounding, not bitwise)
        assert (out_p.float() - eager_p.float()).abs().max().item() <= 4e-3, i
        assert (out_s.float() - eager_s.float()).abs().max().item() <= 4e-3, i
        assert np.abs(out_p.float().cpu().numpy() - ref_p).max() <= TOL[wl.dtype], i
        assert np.abs(out_s.float().cpu().numpy() - ref_s).max() <= TOL[wl.dtype], i
    assert gb.fault() == 0


def test_fp32_repeat_calls_are_bit_identical(A):
    """The fp32 kernel assigns pages to waves statically: same inputs, same bits."""
    wl = W.random_small(132, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4, batch=3)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    step = gb.parallel(ones)
    q = wl.draw_q(step.NQ).to(gb.dev)
    a = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace).clone()
    b = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace)
    assert torch.equal(a, b)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_softmax_scale_argument(A, dtype):
    """sm_scale other than the default: scores scaled by c / sqrt(head_dim) with queries q are the scores
    of the default scale with queries c q, which is what the oracle is given (c a power of two, so that
    c q is exact in either dtype)."""
    kw = dict(dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=2) if dtype == "f32" else {}
    wl = W.random_small(141, batch=3, **kw)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    q = wl.draw_q(meta.NQ)
    for c in (0.25, 2.0):
        ref, ref_lse = attend(tt, meta, q * c, wl.k_cache, wl.v_cache)
        lse = torch.full((meta.NQ, wl.num_q_heads), float("nan"), dtype=torch.float32, device=gb.dev)
        out = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace, lse=lse,
                                          sm_scale=c / math.sqrt(wl.head_dim))
        torch.cuda.synchronize()
        assert np.abs(out.float().cpu().numpy() - ref).max() <= TOL[wl.dtype], c
        assert np.abs(lse.cpu().numpy() - ref_lse).max() <= LSE_TOL[wl.dtype], c


def test_hint_does_not_change_results(A):
    """max_new_per_seq only sizes the row tile: a wrong or missing hint gives the same result."""
    wl = W.random_small(133, batch=3, branches_range=(5, 7))
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    q = wl.draw_q(meta.NQ)
    ref, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache)
    for hint in (0, 1, 2, 7, 100):
        step.max_new_per_seq = hint
        out = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace)
        err = np.abs(out.float().cpu().numpy() - ref).max()
        assert err <= TOL[wl.dtype], (hint, err)


# --------------------------------------------------------------------------------------------- seeded sweep
def test_seeded_sweep_on_a_shared_workspace(A):
    """Forty seeded random shapes (dtype, head sizes, batch, prefix, branches), every call kind, each
    launch three times in a row on ONE workspace shared by all shapes: a launch meets the records of
    the launch before it, of another call kind and of another batch."""
    from gpu_drive import GpuBatch, assert_step_equal, assert_state_equal
    ws = torch.zeros(200 << 20, dtype=torch.uint8, device="cuda")
    A.aspd_workspace_init(ws)
    for seed in range(7001, 7041):
        rng = np.random.default_rng(seed)
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        D = int(rng.choice([64, 128]))
        if dtype == "f32":
            Hkv, G = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4]))
        else:
            Hkv, G = int(rng.choice([1, 2, 8])), int(rng.choice([1, 2, 4, 8, 16]))
        B = int(rng.integers(1, 9))
        pmax = int(rng.choice([10, 100, 700, 3000, 9000]))
        kb = int(rng.choice([1, 3, 8, 20]))
        wl = W.random_small(seed=seed, dtype=dtype, head_dim=D, num_q_heads=Hkv * G, num_kv_heads=Hkv, batch=B,
                            prefix_range=(0, pmax), branches_range=(1, kb),
                            branch_len_range=(1, int(rng.choice([3, 20, 70]))), extra_tokens_per_branch=24,
                            extra_tokens_per_seq=12)
        label = f"seed {seed} {dtype} D{D} Hkv{Hkv} G{G} B{B} pmax{pmax} K<={kb}"
        gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
        gb.workspace = ws

        def check(meta, step, fn, what, hint):
            assert_step_equal(step, meta)
            q = wl.draw_q(meta.NQ)
            step.max_new_per_seq = hint
            ref, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache)
            for rep in range(3):
                out = fn(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace)
                err = np.abs(out.float().cpu().numpy().astype(np.float64) - ref).max()
                assert np.isfinite(err) and err <= TOL[dtype], (label, what, rep, err)

        ones = np.ones(wl.NB, dtype=np.int32)
        check(tt.append_parallel(ones), gb.parallel(ones), A.aspd_attn_parallel_decode, "parallel",
              int(rng.choice([0, int(wl.num_branches.max())])))
        ch = rng.integers(0, int(rng.choice([3, 9, 21])), size=wl.NB).astype(np.int32)
        if ch.sum():
            check(tt.append_parallel(ch), gb.parallel(ch), A.aspd_attn_branch_chunk, "chunk", 0)
        tt.merge()
        gb.merge()
        nm = rng.integers(0, int(rng.choice([2, 2, 30])), size=wl.B).astype(np.int32)
        if nm.sum() and (nm <= 12).all():
            check(tt.append_serial(nm), gb.serial(nm), A.aspd_attn_serial_decode, "serial",
                  int(rng.choice([0, int(nm.max())])))
        assert_state_equal(gb, tt)


# --------------------------------------------------------------------------------------------- degenerate inputs
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_without_tokens_is_a_no_op(A, dtype):
    """Every branch finished (new_len all zero): the metadata call leaves the state as it is and the
    attention calls return without touching their output."""
    from gpu_drive import assert_state_equal
    kw = dict(dtype=dtype, head_dim=64, num_q_heads=4, num_kv_heads=4 if dtype == "f32" else 2, batch=3)
    wl = W.random_small(151, **kw)
    gb, tt = _grow_both(A, wl, wl.branch_len, False)
    zeros = np.zeros(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(zeros)
    step = gb.parallel(zeros)
    assert step.NQ == 0 and meta.NQ == 0
    assert gb.fault() == 0
    assert_state_equal(gb, tt)
    q = torch.zeros(1, wl.num_q_heads, wl.head_dim, dtype=wl.torch_dtype, device=gb.dev)
    out = torch.full_like(q, 7.0)
    for fn in (A.aspd_attn_parallel_decode, A.aspd_attn_branch_chunk):
        fn(gb.kv, gb.state, step, q, gb.workspace, out=out)
    torch.cuda.synchronize()
    assert (out == 7.0).all()


def test_single_branch_is_plain_causal_attention(A):
    """K = 1: the branch sees the prefix and itself, which is ordinary causal attention; checked against
    torch's own scaled-dot-product attention (a second reference besides the oracle)."""
    wl = W.random_small(152, dtype="bf16", head_dim=128, num_q_heads=8, num_kv_heads=2, batch=2,
                        prefix_range=(100, 900), branches_range=(1, 1), branch_len_range=(5, 40))
    gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
    ones = np.ones(wl.NB, dtype=np.int32)
    meta = tt.append_parallel(ones)
    step = gb.parallel(ones)
    _compare_attention(A, gb, tt, wl, step, meta, A.aspd_attn_parallel_decode, label="single branch")
    # the same through torch: the query of sequence s attends every token of s
    q = wl.draw_q(meta.NQ)
    out = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q.to(gb.dev), gb.workspace).float().cpu()
    G = wl.num_q_heads // wl.num_kv_heads
    for s in range(wl.B):
        phys = torch.from_numpy(np.asarray(tt.physical_slots(s), dtype=np.int64))
        k = wl.k_cache[phys // 16, :, phys % 16].float()          # [T][Hkv][D]
        v = wl.v_cache[phys // 16, :, phys % 16].float()
        k = k.permute(1, 0, 2).repeat_interleave(G, dim=0)         # [Hq][T][D]
        v = v.permute(1, 0, 2).repeat_interleave(G, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(q[s].float().unsqueeze(1), k, v)  # [Hq][1][D]
        assert (out[s] - ref[:, 0]).abs().max().item() <= TOL["bf16"]


# --------------------------------------------------------------------------------------------- faults (host-forced)
def test_outgrowing_the_block_table_raises_a_fault_and_writes_nothing(A):
    from gpu_drive import GpuBatch
    wl = W.random_small(140, batch=2, extra_tokens_per_branch=0, extra_tokens_per_seq=0)
    gb = GpuBatch(wl)
    gb.grow_to(wl.branch_len)
    assert gb.fault() == 0
    before = gb.state.seq_len.clone()
    big = np.full(wl.NB, 64, dtype=np.int32)     # far beyond the capacity of every sequence
    step = gb.parallel(big)
    torch.cuda.synchronize()
    assert gb.fault() & A.FAULT_BLOCK_TABLE
    assert torch.equal(gb.state.seq_len, before)


def test_row_count_mismatch_raises_a_fault(A):
    from gpu_drive import GpuBatch
    wl = W.random_small(141, batch=2)
    gb = GpuBatch(wl)
    gb.serial(wl.prefix_len)
    gb.open_parallel()
    ones = np.ones(wl.NB, dtype=np.int32)
    new_len = torch.from_numpy(ones).to(gb.dev)
    A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_PARALLEL, new_len, NQ=max(wl.NB - 1, 0) or 1)
    torch.cuda.synchronize()
    if wl.NB > 1:
        assert gb.fault() & A.FAULT_ROW_COUNT


def test_two_streams_two_workspaces(A):
    """Two batches decoded at the same time on two streams (default priority), each call with its own workspace, as
    the header allows; both against the oracle and against the same calls issued one after the other."""
    wl1 = W.config(3, scale=0.2, batch=6)
    wl2 = W.random_small(seed=777, batch=5, prefix_range=(500, 1500), branches_range=(2, 6), branch_len_range=(10, 60))
    sides = []
    for wl in (wl1, wl2):
        gb, tt = _grow_both(A, wl, wl.branch_len - 1, False)
        ones = np.ones(wl.NB, dtype=np.int32)
        meta = tt.append_parallel(ones)
        step = gb.parallel(ones)
        q = wl.draw_q(meta.NQ)
        ref, _ = attend(tt, meta, q, wl.k_cache, wl.v_cache)
        sides.append((wl, gb, step, q.to(gb.dev), ref))
    torch.cuda.synchronize()
    serial = [A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace).clone() for _, gb, step, q, _ in sides]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.empty_like(s) for s in serial]
    for rep in range(6):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        for (wl, gb, step, q, _), st, o in zip(sides, streams, outs):
            with torch.cuda.stream(st):
                for _ in range(4):      # several launches each, so that the two streams do overlap
                    A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace, out=o)
        torch.cuda.synchronize()
        for (wl, gb, step, q, ref), o, s in zip(sides, outs, serial):
            assert np.abs(o.float().cpu().numpy() - ref).max() <= TOL[wl.dtype], rep
            assert (o.float() - s.float()).abs().max().item() <= 4e-3, rep
