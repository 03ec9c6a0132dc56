"""The shared library loads, exports every symbol the header declares, and rejects bad arguments
on the host before anything would be launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2508_08895_amd import binding as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "aspd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aspd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(A.EXPORTS)
    L = A.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert A.status_string(A.OK) == "ok"
    for code in (A.ERR_INVALID_ARG, A.ERR_UNSUPPORTED, A.ERR_WORKSPACE, A.ERR_HIP):
        assert A.status_string(code) not in ("ok", "unknown status")
    assert A.status_string(-99) == "unknown status"


def _kv(**over):
    base = dict(k_cache_d=0x1000, v_cache_d=0x2000, block_tables_d=0x3000, num_blocks=8, block_size=16,
                num_q_heads=32, num_kv_heads=8, head_dim=128, max_blocks_per_seq=4, dtype=A.BF16)
    base.update(over)
    return A.aspd_kv(**base)


def test_workspace_init_rejects_bad_arguments():
    L = A.lib()
    assert L.aspd_workspace_init(None, 1 << 20, None) == A.ERR_INVALID_ARG
    assert L.aspd_workspace_init(0x1010, 1 << 20, None) == A.ERR_INVALID_ARG
    assert L.aspd_workspace_init(0x1000, 16, None) == A.ERR_WORKSPACE


def test_workspace_bytes_is_host_only():
    L = A.lib()
    kv = _kv()
    n = L.aspd_workspace_bytes(C.byref(kv), 4, 16)
    assert n > 0 and n % 16 == 0
    assert L.aspd_workspace_bytes(C.byref(_kv(head_dim=96)), 4, 16) == 0
    assert L.aspd_workspace_bytes(C.byref(kv), 0, 16) == 0
    assert L.aspd_workspace_bytes(None, 4, 16) == 0
    # fp32 rows are fewer: smaller scratch
    assert L.aspd_workspace_bytes(C.byref(_kv(dtype=A.F32)), 4, 16) < n


@pytest.mark.parametrize("over,code", [
    (dict(k_cache_d=None), A.ERR_INVALID_ARG),
    (dict(block_size=32), A.ERR_UNSUPPORTED),
    (dict(head_dim=96), A.ERR_UNSUPPORTED),
    (dict(num_q_heads=30), A.ERR_UNSUPPORTED),
    (dict(dtype=7), A.ERR_UNSUPPORTED),
    (dict(k_cache_d=0x1004), A.ERR_INVALID_ARG),
    (dict(num_blocks=0), A.ERR_INVALID_ARG),
])
def test_bad_cache_descriptors_are_rejected_before_launch(over, code):
    L = A.lib()
    kv = _kv(**over)
    st = A.aspd_state(B=1, NB=1, stage_base_d=0x10, seq_len_d=0x20, cu_branches_d=0x30, branch_len_d=0x40,
                      slot_owner_d=0x50, owner_stride=64, fault_d=None)
    sp = A.aspd_step(NQ=1, max_new_per_seq=0, cu_new_d=0x10, cu_seq_new_d=0x10, q_seq_d=0x10, q_branch_d=0x10,
                     position_ids_d=0x10, logical_slot_d=0x10, slot_mapping_d=0x10, kv_len_d=0x10)
    assert L.aspd_build_branch_meta(C.byref(kv), C.byref(st), A.STAGE_PARALLEL, 0, 0x100, C.byref(sp), None) == code
    for name in ("aspd_attn_parallel_decode", "aspd_attn_branch_chunk", "aspd_attn_serial_decode"):
        rc = getattr(L, name)(C.byref(kv), C.byref(st), C.byref(sp), 0x100, 0x200, None, 0.0, 0x300, 1 << 30, None)
        assert rc == code, name


def test_bad_state_and_step_are_rejected_before_launch():
    L = A.lib()
    kv = _kv()
    good_st = dict(B=1, NB=1, stage_base_d=0x10, seq_len_d=0x20, cu_branches_d=0x30, branch_len_d=0x40,
                   slot_owner_d=0x50, owner_stride=64, fault_d=None)
    good_sp = dict(NQ=1, max_new_per_seq=0, cu_new_d=0x10, cu_seq_new_d=0x10, q_seq_d=0x10, q_branch_d=0x10, position_ids_d=0x10,
                   logical_slot_d=0x10, slot_mapping_d=0x10, kv_len_d=0x10)

    def meta(st_over=None, sp_over=None, stage=A.STAGE_PARALLEL, pos=0, new_len=0x100):
        st = A.aspd_state(**{**good_st, **(st_over or {})})
        sp = A.aspd_step(**{**good_sp, **(sp_over or {})})
        return L.aspd_build_branch_meta(C.byref(kv), C.byref(st), stage, pos, new_len, C.byref(sp), None)

    assert meta(st_over=dict(B=0)) == A.ERR_INVALID_ARG
    assert meta(st_over=dict(B=5000)) == A.ERR_UNSUPPORTED
    assert meta(st_over=dict(seq_len_d=None)) == A.ERR_INVALID_ARG
    assert meta(st_over=dict(slot_owner_d=None)) == A.ERR_INVALID_ARG
    assert meta(sp_over=dict(NQ=-1)) == A.ERR_INVALID_ARG
    assert meta(sp_over=dict(kv_len_d=None)) == A.ERR_INVALID_ARG
    assert meta(stage=9) == A.ERR_INVALID_ARG
    assert meta(pos=3) == A.ERR_UNSUPPORTED
    assert meta(pos=A.POS_SAME_MAX) == A.ERR_INVALID_ARG                     # needs state.main_pos_d
    assert meta(pos=A.POS_FIX_N(32), st_over=dict(main_pos_d=None)) == A.ERR_INVALID_ARG
    assert meta(pos=2) == A.ERR_UNSUPPORTED                                  # fixed intervals of 0 positions
    assert meta(new_len=None) == A.ERR_INVALID_ARG

    def attn(st_over=None, sp_over=None, q=0x100, out=0x200, ws=0x300, ws_bytes=1 << 30, scale=0.0,
             name="aspd_attn_parallel_decode"):
        st = A.aspd_state(**{**good_st, **(st_over or {})})
        sp = A.aspd_step(**{**good_sp, **(sp_over or {})})
        return getattr(L, name)(C.byref(kv), C.byref(st), C.byref(sp), q, out, None, scale, ws, ws_bytes, None)

    assert attn(q=None) == A.ERR_INVALID_ARG
    assert attn(q=0x104) == A.ERR_INVALID_ARG
    assert attn(ws=None) == A.ERR_INVALID_ARG
    assert attn(ws=0x310) == A.ERR_INVALID_ARG
    assert attn(ws_bytes=1024) == A.ERR_WORKSPACE
    assert attn(scale=-1.0) == A.ERR_INVALID_ARG
    assert attn(st_over=dict(owner_stride=16)) == A.ERR_INVALID_ARG      # below max_blocks_per_seq * 16
    assert attn(st_over=dict(slot_owner_d=None)) == A.ERR_INVALID_ARG
    assert attn(st_over=dict(slot_owner_d=None), name="aspd_attn_serial_decode", q=None) == A.ERR_INVALID_ARG
    assert attn(sp_over=dict(NQ=0), q=None) == A.OK                        # nothing to do, nothing launched
    # group wider than the row tile
    kv_wide = _kv(num_q_heads=64, num_kv_heads=1, dtype=A.F32)
    st = A.aspd_state(**good_st)
    sp = A.aspd_step(**good_sp)
    rc = L.aspd_attn_parallel_decode(C.byref(kv_wide), C.byref(st), C.byref(sp), 0x100, 0x200, None, 0.0, 0x300,
                                     1 << 30, None)
    assert rc == A.ERR_UNSUPPORTED


def test_rope_append_and_renumber_reject_bad_arguments_before_launch():
    L = A.lib()
    kv = _kv()
    sp = dict(NQ=1, max_new_per_seq=0, cu_new_d=0x10, cu_seq_new_d=0x10, q_seq_d=0x10, q_branch_d=0x10,
              position_ids_d=0x10, logical_slot_d=0x10, slot_mapping_d=0x10, kv_len_d=0x10)

    def rope(kv_=kv, sp_over=None, q=0x100, k=0x200, v=0x300, theta=10000.0):
        s = A.aspd_step(**{**sp, **(sp_over or {})})
        return L.aspd_rope_append(C.byref(kv_), C.byref(s), q, k, v, theta, None)

    assert rope(kv_=_kv(head_dim=96)) == A.ERR_UNSUPPORTED
    assert rope(q=None) == A.ERR_INVALID_ARG
    assert rope(k=None) == A.ERR_INVALID_ARG
    assert rope(v=None) == A.ERR_INVALID_ARG
    assert rope(theta=1.0) == A.ERR_INVALID_ARG
    assert rope(theta=float("nan")) == A.ERR_INVALID_ARG
    assert rope(sp_over=dict(NQ=-2)) == A.ERR_INVALID_ARG
    assert rope(sp_over=dict(slot_mapping_d=None)) == A.ERR_INVALID_ARG
    assert rope(sp_over=dict(NQ=0), q=None) == A.OK            # nothing to do, nothing launched

    st = dict(B=2, NB=1, stage_base_d=0x10, seq_len_d=0x20, cu_branches_d=0x30, branch_len_d=0x40,
              slot_owner_d=0x50, owner_stride=64, fault_d=None)

    def renumber(st_over=None, new_cu=0x400, new_len=0x500):
        s = A.aspd_state(**{**st, **(st_over or {})})
        return L.aspd_renumber_branches(C.byref(s), new_cu, new_len, None)

    assert renumber(new_cu=None) == A.ERR_INVALID_ARG
    assert renumber(new_len=None) == A.ERR_INVALID_ARG
    assert renumber(new_cu=0x30) == A.ERR_INVALID_ARG          # must not be the array in use
    assert renumber(new_len=0x40) == A.ERR_INVALID_ARG
    assert renumber(st_over=dict(B=0)) == A.ERR_INVALID_ARG
    assert renumber(st_over=dict(cu_branches_d=None)) == A.ERR_INVALID_ARG


def test_assembly_that_may_read_mfma_results_brings_its_wait_states():
    """The matrix unit does not interlock with a vector or memory instruction that reads an MFMA result too
    soon, and the compiler pads only the instructions it emits itself.  Every inline-assembly statement of the
    kernels that contains a vector or memory instruction with register inputs must therefore start with its own
    wait states (`s_nop 15`), so that it is safe wherever the scheduler puts it."""
    import glob, os, re
    here = os.path.dirname(os.path.abspath(__file__))
    files = sorted(glob.glob(os.path.join(here, "..", "paper_2508_08895_amd", "csrc", "*.h")) +
                   glob.glob(os.path.join(here, "..", "paper_2508_08895_amd", "csrc", "*.hip")))
    assert files
    seen = 0
    for f in files:
        src = open(f).read()
        for m in re.finditer(r"\basm\s*(?:volatile)?\s*\(", src):
            # the statement up to its closing parenthesis + semicolon
            depth, i = 0, m.end() - 1
            while True:
                depth += src[i] == "("
                depth -= src[i] == ")"
                i += 1
                if depth == 0:
                    break
            stmt = src[m.start():i]
            text = "".join(re.findall(r'"((?:[^"\\]|\\.)*)"', stmt.split(":")[0]))
            text = text.replace("\\n", " ").replace("\\t", " ")
            if not re.search(r"\b(v_[a-z0-9_]+|global_store_[a-z0-9]+|ds_write_[a-z0-9]+)\b", text):
                continue
            seen += 1
            assert text.lstrip().startswith("s_nop 15"), (os.path.basename(f), text[:60])
    assert seen >= 2   # the three-operand maximum and the write-through store
