"""The C writing of the oracle's attention (oracle/attention_ref.c) against the same pins as the numpy one,
and the two against each other."""
import numpy as np
import pytest

import aspd_workloads as W
import test_oracle_attention as T
from oracle import attend
from oracle.attention_c import attend_c
from oracle_drive import table_at


@pytest.fixture(autouse=True)
def _pins_run_on_the_c_oracle(monkeypatch):
    monkeypatch.setattr(T, "attend", attend_c)


test_zero_queries_give_mean_of_visible_values = T.test_zero_queries_give_mean_of_visible_values
test_single_visible_key_returns_its_value = T.test_single_visible_key_returns_its_value
test_equal_values_pass_through = T.test_equal_values_pass_through
test_single_branch_equals_library_causal_attention = T.test_single_branch_equals_library_causal_attention
test_sibling_perturbation_leaves_output_bit_identical = T.test_sibling_perturbation_leaves_output_bit_identical
test_branch_permutation_permutes_outputs = T.test_branch_permutation_permutes_outputs
test_serial_after_merge_equals_unmasked_attention_over_all_rows = T.test_serial_after_merge_equals_unmasked_attention_over_all_rows
test_weights_shift_invariance_and_lse = T.test_weights_shift_invariance_and_lse


@pytest.mark.parametrize("seed,kw", [(301, {}), (302, dict(dtype="f32", head_dim=64, num_q_heads=4, num_kv_heads=2))])
def test_the_two_writings_agree(seed, kw):
    wl = W.random_small(seed, batch=3, **kw)
    tt = table_at(wl, wl.branch_len)
    for new_len in (np.ones(wl.NB, dtype=np.int32), np.full(wl.NB, 3, dtype=np.int32)):
        m = tt.append_parallel(new_len)
        q = wl.draw_q(m.NQ)
        a, la = attend(tt, m, q, wl.k_cache, wl.v_cache)
        b, lb = attend_c(tt, m, q, wl.k_cache, wl.v_cache)
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
        np.testing.assert_allclose(la, lb, rtol=0, atol=1e-12)
        c, _ = attend_c(tt, m, q, wl.k_cache, wl.v_cache, shared_mask=True)
        d, _ = attend(tt, m, q, wl.k_cache, wl.v_cache, shared_mask=True)
        np.testing.assert_allclose(c, d, rtol=0, atol=1e-13)
