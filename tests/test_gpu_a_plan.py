"""The step's attention plan (written by aspd_build_branch_meta next to the metadata) read back and checked
on the host, before any attention kernel consumes one: every (sequence, row group, KV head) item's pages
are covered exactly once, by consecutive workgroups, each with one run; the workgroups named as first and
last holder of an item are the ones that hold its first and last page; the block ids in a header are
the block table's; every field stays inside the call's arrays.  Layout as documented in csrc/aspd_plan.h."""
import numpy as np
import pytest
import torch

import aspd_workloads as W

pytestmark = pytest.mark.gpu

HDR, SEG, NSEG, NEXT, IDS = 32, 8, 8, 9, 16


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_08895_amd import binding
    binding.lib()
    return binding


def _decode_key(key):
    B = key % 1024
    pad = (key >> 10) % 256
    qpg = (key >> 18) % 512
    nwg = (key >> 27) % 2048
    return B, pad, qpg, nwg


def _check_plan(gb, step, label):
    wl = gb.wl
    assert step.plan_key != 0, label
    B, pad, qpg, nwg = _decode_key(step.plan_key)
    assert B == wl.B and 1 <= nwg <= 1024 and qpg >= 1
    plan = step.plan.cpu().numpy().view(np.int32)
    T = gb.state.seq_len.cpu().numpy()
    L = gb.state.stage_base.cpu().numpy()
    cu = step.cu_seq_new.cpu().numpy()
    bt = wl.block_tables
    Hkv = wl.num_kv_heads
    pieces = {}          # (s, h, q0) -> list of (workgroup, page0, page1, np, owner, w_last, nq)
    total_extra = 0
    for w in range(nwg):
        hdr = plan[HDR * w: HDR * (w + 1)]
        nseg, nxt = int(hdr[NSEG]), int(hdr[NEXT])
        assert nseg >= 0
        assert nxt == total_extra, (label, w)          # extras are laid out in workgroup order
        total_extra += max(nseg - 1, 0)
        for i in range(nseg):
            d = hdr[:SEG] if i == 0 else plan[HDR * nwg + SEG * (nxt + i - 1): HDR * nwg + SEG * (nxt + i)]
            s, h = int(d[0]) & 0xffff, int(np.uint32(d[0]) >> 16)
            q0, nq, p0, p1, npg = (int(x) for x in d[1:6])
            owner, w_last = int(d[6]) & 0xffff, int(np.uint32(d[6]) >> 16)
            assert 0 <= s < wl.B and 0 <= h < Hkv, (label, w, i)
            assert npg == min((T[s] + 15) // 16, bt.shape[1])
            assert 0 <= p0 < p1 <= npg
            assert cu[s] <= q0 and 1 <= nq <= qpg and q0 + nq <= cu[s + 1]
            assert (q0 - cu[s]) % qpg == 0 and (nq == qpg or q0 + nq == cu[s + 1])
            assert int(d[7]) == L[s]
            assert owner <= w <= w_last < nwg
            pieces.setdefault((s, h, q0), []).append((w, p0, p1, owner, w_last))
            if i == 0:
                want = [bt[s, min(p0 + k, p1 - 1)] for k in range(16)]
                assert hdr[IDS:IDS + 16].tolist() == want, (label, w)
    # every item is covered exactly once
    items = 0
    for s in range(wl.B):
        nq_s = int(cu[s + 1] - cu[s])
        npg = min((T[s] + 15) // 16, bt.shape[1])
        if nq_s == 0 or npg == 0:
            continue
        for h in range(Hkv):
            for q0 in range(int(cu[s]), int(cu[s + 1]), qpg):
                items += 1
                runs = pieces.pop((s, h, q0), None)
                assert runs, (label, s, h, q0)
                runs.sort()
                assert runs[0][1] == 0 and runs[-1][2] == npg, (label, s, h, q0, runs)
                for a, b in zip(runs, runs[1:]):
                    assert a[2] == b[1] and b[0] == a[0] + 1, (label, s, h, q0, runs)   # consecutive pages, consecutive workgroups
                for r in runs:
                    assert r[3] == runs[0][0] and r[4] == runs[-1][0], (label, s, h, q0, runs)
    assert not pieces, (label, list(pieces)[:4])
    return items, nwg


def _grown(A, wl, upto):
    from gpu_drive import GpuBatch
    gb = GpuBatch(wl)
    gb.grow_to(upto)
    assert gb.fault() == 0
    return gb


@pytest.mark.parametrize("case", ["cfg2", "cfg3", "cfg4", "cfg5_eighth", "batch150", "small", "f32", "capped"])
def test_plan_covers_every_item_once(A, case):
    hint_chunk = None
    cap = 0
    if case == "cfg2":
        wl = W.config(2)
    elif case == "cfg3":
        wl = W.config(3)
    elif case == "cfg4":
        wl = W.config(4, scale=0.25)
    elif case == "cfg5_eighth":
        wl = W.config(5, scale=0.125, batch=8)
    elif case == "batch150":
        wl = W.config(3, scale=0.06, batch=150)
    elif case == "small":
        wl = W.random_small(seed=901, batch=5, branches_range=(1, 12))
    elif case == "f32":
        wl = W.random_small(seed=902, dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=2, batch=4,
                            prefix_range=(0, 900))
    else:
        wl = W.random_small(seed=903, batch=3, prefix_range=(2000, 5000))
        cap = 5
    upto = np.minimum(wl.branch_len, 24) if case == "batch150" else wl.branch_len
    gb = _grown(A, wl, upto - 1)
    K = int(wl.num_branches.max())
    # decode step, with the hint a decoding loop gives and without
    for hint in (K, 0):
        st = [t.clone() for t in (gb.state.stage_base, gb.state.seq_len, gb.state.branch_len)]
        ones = np.ones(wl.NB, dtype=np.int32)
        step = A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_PARALLEL, gb._dev_i32(ones), NQ=wl.NB,
                                        max_new_per_seq=hint, max_workgroups=cap)
        torch.cuda.synchronize()
        items, nwg = _check_plan(gb, step, f"{case} decode hint {hint}")
        print(f"[{case}] decode hint {hint}: {items} items over {nwg} workgroups", flush=True)
        for dst, src in zip((gb.state.stage_base, gb.state.seq_len, gb.state.branch_len), st):
            dst.copy_(src)
    # a chunk that the row-splitting kernel takes
    chunk = np.full(wl.NB, 5, dtype=np.int32)
    fits = (gb.state.seq_len.cpu().numpy() + 5 * wl.num_branches <= 16 * (wl.block_tables >= 0).sum(axis=1)).all()
    if fits:
        step = A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_PARALLEL, gb._dev_i32(chunk), NQ=5 * wl.NB,
                                        max_new_per_seq=5 * K, max_workgroups=cap)
        torch.cuda.synchronize()
        assert gb.fault() == 0
        _check_plan(gb, step, f"{case} chunk")
    # merge, serial step
    gb.merge()
    one = np.ones(wl.B, dtype=np.int32)
    fits = (gb.state.seq_len.cpu().numpy() + 1 <= 16 * (wl.block_tables >= 0).sum(axis=1)).all()
    if fits:
        step = A.aspd_build_branch_meta(gb.kv, gb.state, A.STAGE_SERIAL, gb._dev_i32(one), NQ=wl.B, max_new_per_seq=1,
                                        max_workgroups=cap)
        torch.cuda.synchronize()
        assert gb.fault() == 0
        _check_plan(gb, step, f"{case} serial")
