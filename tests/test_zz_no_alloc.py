"""aspd_attn_parallel_decode_static (the entry point that allocates nothing) against
aspd_attn_parallel_decode, through the C ABI: two calls in a row on the library's static scratch, the
second with a smaller input, then a call that does not fit."""
import numpy as np
import pytest
import torch

import aspd_workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_08895_amd import binding
    binding.lib()
    return binding


def _batch_at_decode_step(A, wl):
    from gpu_drive import GpuBatch
    gb = GpuBatch(wl)
    gb.grow_to(wl.branch_len - 1)
    ones = np.ones(wl.NB, dtype=np.int32)
    step = gb.parallel(ones)
    step.max_new_per_seq = int(wl.num_branches.max())
    assert gb.fault() == 0
    return gb, step


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_matches_the_workspace_call_twice_in_a_row(A, dtype):
    kw = dict(dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=4) if dtype == "f32" else {}
    big = W.random_small(seed=811, batch=5, prefix_range=(3000, 9000), branches_range=(2, 6),
                         branch_len_range=(3, 30), **kw)
    small = W.random_small(seed=812, batch=2, prefix_range=(10, 200), branches_range=(1, 3),
                           branch_len_range=(2, 9), **kw)
    for wl in (big, small):           # the second call meets what the first left in the scratch
        gb, step = _batch_at_decode_step(A, wl)
        q = wl.draw_q(step.NQ).to(gb.dev)
        lse_ws = torch.full((step.NQ, wl.num_q_heads), float("nan"), dtype=torch.float32, device=gb.dev)
        lse_st = lse_ws.clone()
        want = A.aspd_attn_parallel_decode(gb.kv, gb.state, step, q, gb.workspace, lse=lse_ws)
        got = torch.full_like(q, float("nan"))
        A.aspd_attn_parallel_decode_static(gb.kv, gb.state, step, q, got, lse=lse_st)
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        if dtype == "f32":            # static page-to-wave assignment: the same bits
            assert torch.equal(got, want) and torch.equal(lse_st, lse_ws)
        else:                         # pairs of pages are handed to waves dynamically: equal to rounding
            assert (got.float() - want.float()).abs().max().item() <= 4e-3
            assert (lse_st - lse_ws).abs().max().item() <= 2e-3
        # and against the oracle, to the tolerance of the parity tests
        from oracle import attend
        from oracle_drive import table_at
        tt = table_at(wl, wl.branch_len - 1)
        meta = tt.append_parallel(np.ones(wl.NB, dtype=np.int32))
        ref, _ = attend(tt, meta, q.cpu(), wl.k_cache, wl.v_cache)
        assert np.abs(got.float().cpu().numpy() - ref).max() <= (1e-5 if dtype == "f32" else 2e-2)


def test_static_scratch_rejects_what_does_not_fit(A):
    """A step whose hint sends it to the row-splitting kernel needs 69 MB of partial slots: refused with
    its own error code, nothing launched, output untouched."""
    wl = W.random_small(seed=813, batch=4, prefix_range=(3000, 4000), branches_range=(20, 20), branch_len_range=(2, 4),
                        num_q_heads=32, num_kv_heads=8)    # pages enough for a full grid of the row-splitting kernel
    gb, step = _batch_at_decode_step(A, wl)
    step.max_new_per_seq = 64           # 64 tokens x 4 heads per KV head: more rows than the streaming kernels take
    q = wl.draw_q(step.NQ).to(gb.dev)
    out = torch.full_like(q, 7.0)
    with pytest.raises(A.AspdError) as e:
        A.aspd_attn_parallel_decode_static(gb.kv, gb.state, step, q, out)
    assert e.value.code == A.ERR_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert (out == 7.0).all()
