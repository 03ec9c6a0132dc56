"""Pins for the oracle's attention (Eq. 1 with the mask of Eq. 2-3).

Closed forms, textbook special cases, a library routine for the cases that reduce to plain
causal / unmasked attention, and the invariants the paper states (branch isolation, branch
symmetry, lossless merge)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import aspd_workloads as W
from oracle import TokenTable, attend
from oracle_drive import table_at, table_with_prefix


def _gather(wl, tt, s, cache):
    """[Hkv][T][D] float64 rows of sequence s in slot order, through the block table (written
    separately from the oracle's own reader)."""
    T = len(tt.pos[s])
    out = torch.empty(wl.num_kv_heads, T, wl.head_dim, dtype=torch.float64)
    for j in range(T):
        blk = int(wl.block_tables[s, j // 16])
        out[:, j] = cache[blk, :, j % 16].to(torch.float64)
    return out


def test_zero_queries_give_mean_of_visible_values():
    # q = 0 => equal weights => output = arithmetic mean of the visible V rows: pins the mask
    # through the whole attention path, with a closed form
    wl = W.random_small(21, batch=3)
    tt = table_at(wl, wl.branch_len - 1) if (wl.branch_len > 1).all() else table_at(wl, wl.branch_len)
    m = tt.append_parallel(np.ones(wl.NB, dtype=np.int32))
    q = torch.zeros(m.NQ, wl.num_q_heads, wl.head_dim, dtype=wl.torch_dtype)
    out, lse = attend(tt, m, q, wl.k_cache, wl.v_cache)
    G = wl.num_q_heads // wl.num_kv_heads
    seq_of_branch = np.repeat(np.arange(wl.B), wl.num_branches)
    cu = wl.cu_branches
    for r in range(m.NQ):
        s = int(m.q_seq[r])
        v = _gather(wl, tt, s, wl.v_cache).numpy()
        L = int(wl.prefix_len[s])
        tag = int(m.q_branch[r]) - int(cu[s]) + 1
        own = [j for j in range(L, len(tt.pos[s])) if tt.branch[s][j] == tag]
        vis = list(range(L)) + own
        assert len(vis) == m.kv_len[r]
        for h in range(wl.num_q_heads):
            np.testing.assert_allclose(out[r, h], v[h // G, vis].mean(axis=0), rtol=0, atol=1e-13)
            np.testing.assert_allclose(lse[r, h], np.log(len(vis)), rtol=0, atol=1e-13)


def test_single_visible_key_returns_its_value():
    # empty prefix, first token of each branch: it sees only itself
    wl = W.random_small(22, batch=2, prefix_range=(0, 0))
    tt = table_with_prefix(wl)
    tt.open_parallel(wl.num_branches)
    m = tt.append_parallel(np.ones(wl.NB, dtype=np.int32))
    assert (m.kv_len == 1).all()
    q = wl.draw_q(m.NQ)
    out, lse = attend(tt, m, q, wl.k_cache, wl.v_cache)
    G = wl.num_q_heads // wl.num_kv_heads
    for r in range(m.NQ):
        ph = int(m.slot_mapping[r])
        for h in range(wl.num_q_heads):
            v = wl.v_cache[ph // 16, h // G, ph % 16].to(torch.float64).numpy()
            k = wl.k_cache[ph // 16, h // G, ph % 16].to(torch.float64).numpy()
            np.testing.assert_allclose(out[r, h], v, rtol=0, atol=0)
            score = float(q[r, h].to(torch.float64).numpy() @ k) / np.sqrt(wl.head_dim)
            np.testing.assert_allclose(lse[r, h], score, rtol=1e-14, atol=1e-14)


def test_equal_values_pass_through():
    wl = W.random_small(23, batch=2)
    row = torch.linspace(-1, 1, wl.head_dim).to(wl.torch_dtype)
    v = wl.v_cache.clone()
    v[:] = row
    tt = table_at(wl, wl.branch_len)
    m = tt.append_parallel(np.ones(wl.NB, dtype=np.int32))
    out, _ = attend(tt, m, wl.draw_q(m.NQ), wl.k_cache, v)
    np.testing.assert_allclose(out, np.broadcast_to(row.to(torch.float64).numpy(), out.shape), rtol=0, atol=1e-14)


@pytest.mark.parametrize("dtype,D,Hq,Hkv", [("f32", 64, 4, 4), ("bf16", 128, 8, 2)])
def test_single_branch_equals_library_causal_attention(dtype, D, Hq, Hkv):
    # K = 1 reduces to plain causal attention over prefix + branch: check a whole chunk of
    # queries against torch's scaled_dot_product_attention in float64
    wl = W.random_small(24, dtype=dtype, head_dim=D, num_q_heads=Hq, num_kv_heads=Hkv, batch=2,
                        branches_range=(1, 1), prefix_range=(3, 40))
    tt = table_with_prefix(wl)
    tt.open_parallel(wl.num_branches)
    c = np.array([7, 12], dtype=np.int32)
    m = tt.append_parallel(c)
    q = wl.draw_q(m.NQ)
    out, _ = attend(tt, m, q, wl.k_cache, wl.v_cache)
    G = Hq // Hkv
    for s in range(wl.B):
        k = _gather(wl, tt, s, wl.k_cache).repeat_interleave(G, dim=0)   # [Hq][T][D]
        v = _gather(wl, tt, s, wl.v_cache).repeat_interleave(G, dim=0)
        T = k.shape[1]
        rows = slice(int(m.cu_new[s]), int(m.cu_new[s + 1]))
        qs = q[rows].to(torch.float64).permute(1, 0, 2)                  # [Hq][c][D]
        causal = torch.ones(T, T, dtype=torch.bool).tril()[T - int(c[s]):]
        ref = F.scaled_dot_product_attention(qs, k, v, attn_mask=causal)
        np.testing.assert_allclose(out[rows], ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_sibling_perturbation_leaves_output_bit_identical():
    wl = W.random_small(25, batch=2, branches_range=(2, 4))
    tt = table_at(wl, wl.branch_len)
    m = tt.append_parallel(np.ones(wl.NB, dtype=np.int32))
    q = wl.draw_q(m.NQ)
    base, base_lse = attend(tt, m, q, wl.k_cache, wl.v_cache)
    cu = wl.cu_branches
    for r in range(m.NQ):
        s = int(m.q_seq[r])
        tag = int(m.q_branch[r]) - int(cu[s]) + 1
        k2, v2 = wl.k_cache.clone(), wl.v_cache.clone()
        for j in range(int(wl.prefix_len[s]), len(tt.pos[s])):
            if tt.branch[s][j] != tag:
                ph = tt.physical_slot(s, j)
                k2[ph // 16, :, ph % 16] = 1e30 if j % 2 else -3e4
                v2[ph // 16, :, ph % 16] = -1e30
        # same call shape for both, so that the library matmul takes the same summation order
        ref, ref_lse = attend(tt, m, q, wl.k_cache, wl.v_cache, rows=[r])
        out, lse = attend(tt, m, q, k2, v2, rows=[r])
        assert np.array_equal(out[r], ref[r]) and np.array_equal(lse[r], ref_lse[r])
        np.testing.assert_allclose(ref[r], base[r], rtol=0, atol=1e-14)


def test_branch_permutation_permutes_outputs():
    # Eq. 3 has no order among branches: build the same branches in a different order
    wl = W.random_small(26, batch=1, branches_range=(4, 4), branch_len_range=(3, 9))
    K = 4
    perm = np.array([2, 0, 3, 1])
    L = int(wl.prefix_len[0])
    Hkv, D = wl.num_kv_heads, wl.head_dim
    # branch contents, independent of any cache layout
    g = torch.Generator().manual_seed(5)
    content = [(torch.randn(int(n), Hkv, D, generator=g).to(wl.torch_dtype),
                torch.randn(int(n), Hkv, D, generator=g).to(wl.torch_dtype)) for n in wl.branch_len]
    q = wl.draw_q(K)

    def run(order):
        lens = wl.branch_len[order]
        tt = table_with_prefix(wl)
        tt.open_parallel(wl.num_branches)
        k, v = wl.k_cache.clone(), wl.v_cache.clone()
        t_of = np.zeros(K, dtype=int)
        last = None
        for new_len in W.interleaved_history(lens):
            last = tt.append_parallel(new_len)
            for r in range(last.NQ):
                b = int(last.q_branch[r])
                ph = int(last.slot_mapping[r])
                k[ph // 16, :, ph % 16] = content[order[b]][0][t_of[b]]
                v[ph // 16, :, ph % 16] = content[order[b]][1][t_of[b]]
                t_of[b] += 1
        # one more step for every branch, query of branch b belongs to original branch order[b]
        m = tt.append_parallel(np.ones(K, dtype=np.int32))
        out, _ = attend(tt, m, q[order], k, v)
        return out, m

    a, ma = run(np.arange(K))
    b, mb = run(perm)
    # the appended token's own K/V comes from the pool slot it landed in; make the comparison
    # independent of it by checking positions and then outputs up to that one key: give both runs
    # the same landing-slot content instead
    assert np.array_equal(mb.position_ids, ma.position_ids[perm])

    def run_fixed(order):
        lens = wl.branch_len[order]
        tt = table_with_prefix(wl)
        tt.open_parallel(wl.num_branches)
        k, v = wl.k_cache.clone(), wl.v_cache.clone()
        t_of = np.zeros(K, dtype=int)
        hist = W.interleaved_history(lens) + [np.ones(K, dtype=np.int32)]
        extra = [(torch.full((Hkv, D), 0.25 * (i + 1)).to(wl.torch_dtype),
                  torch.full((Hkv, D), -0.5 * (i + 1)).to(wl.torch_dtype)) for i in range(K)]
        for step, new_len in enumerate(hist):
            last = tt.append_parallel(new_len)
            for r in range(last.NQ):
                bb = int(last.q_branch[r])
                ph = int(last.slot_mapping[r])
                src = content[order[bb]]
                if t_of[bb] < src[0].shape[0]:
                    k[ph // 16, :, ph % 16] = src[0][t_of[bb]]
                    v[ph // 16, :, ph % 16] = src[1][t_of[bb]]
                else:
                    k[ph // 16, :, ph % 16] = extra[order[bb]][0]
                    v[ph // 16, :, ph % 16] = extra[order[bb]][1]
                t_of[bb] += 1
        out, _ = attend(tt, last, q[order], k, v)
        return out

    a = run_fixed(np.arange(K))
    b = run_fixed(perm)
    np.testing.assert_allclose(b, a[perm], rtol=0, atol=1e-12)


def test_serial_after_merge_equals_unmasked_attention_over_all_rows():
    # main-branch token after the merge attends the complete history (Sec. 3.2, "The Main
    # Branch's Perspective"): equal to unmasked attention over prefix || branch 1 || ... || branch K
    # gathered separately, in an order different from the cache's
    wl = W.random_small(27, batch=3, extra_tokens_per_seq=2)
    tt = table_at(wl, wl.branch_len)
    tt.merge()
    m = tt.append_serial(np.ones(wl.B, dtype=np.int32))
    q = wl.draw_q(m.NQ)
    out, _ = attend(tt, m, q, wl.k_cache, wl.v_cache)
    G = wl.num_q_heads // wl.num_kv_heads
    for s in range(wl.B):
        T = len(tt.pos[s])
        L = int(wl.prefix_len[s])
        order = list(range(L))
        for tag in range(1, int(wl.num_branches[s]) + 1):       # branch after branch, not interleaved
            order += [j for j in range(L, T - 1) if tt.branch[s][j] == tag]
        order = [T - 1] + order[::-1]                          # and reversed, with the query's key first
        assert sorted(order) == list(range(T))
        k = _gather(wl, tt, s, wl.k_cache)[:, order].repeat_interleave(G, dim=0)
        v = _gather(wl, tt, s, wl.v_cache)[:, order].repeat_interleave(G, dim=0)
        qs = q[s].to(torch.float64)[:, None, :]
        ref = F.scaled_dot_product_attention(qs, k, v)
        np.testing.assert_allclose(out[s], ref[:, 0].numpy(), rtol=0, atol=1e-12)


def test_weights_shift_invariance_and_lse():
    # softmax is invariant to adding a constant to every score: scaling q by 0 gives lse = log n,
    # and lse differences reproduce the weight of a known key
    wl = W.random_small(28, batch=1, branches_range=(2, 2), head_dim=64, num_q_heads=4, num_kv_heads=4,
                        dtype="f32")
    tt = table_at(wl, wl.branch_len)
    m = tt.append_parallel(np.ones(wl.NB, dtype=np.int32))
    q = wl.draw_q(m.NQ)
    out1, lse1 = attend(tt, m, q, wl.k_cache, wl.v_cache, scale=0.125)
    # same scores if q is doubled and the scale halved
    out2, lse2 = attend(tt, m, (q * 2), wl.k_cache, wl.v_cache, scale=0.0625)
    np.testing.assert_allclose(out1, out2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse1, lse2, rtol=0, atol=1e-13)
    # default scale is 1/sqrt(head_dim) = 0.125 for D = 64
    out3, _ = attend(tt, m, q, wl.k_cache, wl.v_cache)
    assert np.array_equal(out1, out3)
