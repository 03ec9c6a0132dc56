"""ctypes binding of libaspd.so: argument marshalling only.

Every operation runs in the library's HIP kernels.  PyTorch is used for device memory
and for the current stream, nothing else.  There is no fallback: if the shared library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaspd.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_SCRATCH_LIMIT = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
STAGE_PARALLEL, STAGE_SERIAL, STAGE_MERGE, STAGE_MIXED = 0, 1, 2, 3
POS_SAME_SEQ, POS_SAME_MAX = 0, 1


def POS_FIX_N(n: int) -> int:
    return 2 | (int(n) << 8)

FAULT_BLOCK_TABLE, FAULT_OWNER_ROW, FAULT_ROW_COUNT, FAULT_BRANCHES, FAULT_STAGE, FAULT_INTERVAL = 1, 2, 4, 8, 16, 32
FAULT_LAYOUT = 64

EXPORTS = ("aspd_build_branch_meta", "aspd_renumber_branches", "aspd_rope_append", "aspd_plan_bytes",
           "aspd_workspace_bytes", "aspd_workspace_init", "aspd_attn_parallel_decode",
           "aspd_attn_branch_chunk", "aspd_attn_serial_decode", "aspd_attn_parallel_decode_static",
           "aspd_sequence_plan_bytes", "aspd_build_sequence_meta", "aspd_attn_full_sequence",
           "aspd_probe_read_bandwidth", "aspd_status_string")


class aspd_kv(C.Structure):
    _fields_ = [("k_cache_d", C.c_void_p), ("v_cache_d", C.c_void_p), ("block_tables_d", C.c_void_p),
                ("num_blocks", C.c_int32), ("block_size", C.c_int32), ("num_q_heads", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("max_blocks_per_seq", C.c_int32),
                ("dtype", C.c_int32)]


class aspd_state(C.Structure):
    _fields_ = [("B", C.c_int32), ("NB", C.c_int32), ("stage_base_d", C.c_void_p), ("seq_len_d", C.c_void_p),
                ("cu_branches_d", C.c_void_p), ("branch_len_d", C.c_void_p), ("slot_owner_d", C.c_void_p),
                ("owner_stride", C.c_int32), ("fault_d", C.c_void_p), ("main_pos_d", C.c_void_p),
                ("stage_open_d", C.c_void_p)]


class aspd_step(C.Structure):
    _fields_ = [("NQ", C.c_int32), ("max_new_per_seq", C.c_int32), ("max_workgroups", C.c_int32),
                ("shared_mask", C.c_int32), ("cu_new_d", C.c_void_p), ("cu_seq_new_d", C.c_void_p),
                ("q_seq_d", C.c_void_p), ("q_branch_d", C.c_void_p), ("position_ids_d", C.c_void_p),
                ("logical_slot_d", C.c_void_p), ("slot_mapping_d", C.c_void_p), ("kv_len_d", C.c_void_p),
                ("plan_d", C.c_void_p), ("plan_bytes", C.c_size_t), ("plan_key", C.c_uint64)]


class aspd_layout(C.Structure):
    _fields_ = [("num_runs", C.c_int32), ("cu_runs_d", C.c_void_p), ("run_branch_d", C.c_void_p),
                ("run_len_d", C.c_void_p)]


class AspdError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {status_string(code)} ({code})")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2508_08895_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.aspd_build_branch_meta.restype = C.c_int
        L.aspd_build_branch_meta.argtypes = [C.POINTER(aspd_kv), C.POINTER(aspd_state), C.c_int32, C.c_int32,
                                             C.c_void_p, C.POINTER(aspd_step), C.c_void_p]
        L.aspd_renumber_branches.restype = C.c_int
        L.aspd_renumber_branches.argtypes = [C.POINTER(aspd_state), C.c_void_p, C.c_void_p, C.c_void_p]
        L.aspd_rope_append.restype = C.c_int
        L.aspd_rope_append.argtypes = [C.POINTER(aspd_kv), C.POINTER(aspd_step), C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_float, C.c_void_p]
        L.aspd_plan_bytes.restype = C.c_size_t
        L.aspd_plan_bytes.argtypes = [C.POINTER(aspd_kv), C.c_int32, C.c_int32]
        L.aspd_workspace_bytes.restype = C.c_size_t
        L.aspd_workspace_bytes.argtypes = [C.POINTER(aspd_kv), C.c_int32, C.c_int32]
        L.aspd_sequence_plan_bytes.restype = C.c_size_t
        L.aspd_sequence_plan_bytes.argtypes = [C.POINTER(aspd_kv), C.c_int32, C.c_int32]
        L.aspd_build_sequence_meta.restype = C.c_int
        L.aspd_build_sequence_meta.argtypes = [C.POINTER(aspd_kv), C.POINTER(aspd_state), C.POINTER(aspd_layout),
                                               C.c_int32, C.POINTER(aspd_step), C.c_void_p]
        for name in ("aspd_attn_parallel_decode", "aspd_attn_branch_chunk", "aspd_attn_serial_decode",
                     "aspd_attn_full_sequence"):
            fn = getattr(L, name)
            fn.restype = C.c_int
            fn.argtypes = [C.POINTER(aspd_kv), C.POINTER(aspd_state), C.POINTER(aspd_step), C.c_void_p,
                           C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
        L.aspd_attn_parallel_decode_static.restype = C.c_int
        L.aspd_attn_parallel_decode_static.argtypes = [C.POINTER(aspd_kv), C.POINTER(aspd_state), C.POINTER(aspd_step),
                                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
        L.aspd_workspace_init.restype = C.c_int
        L.aspd_workspace_init.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        L.aspd_probe_read_bandwidth.restype = C.c_int
        L.aspd_probe_read_bandwidth.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.aspd_status_string.restype = C.c_char_p
        L.aspd_status_string.argtypes = [C.c_int]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().aspd_status_string(int(code)).decode()


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


_DTYPE = {torch.float32: F32, torch.bfloat16: BF16}


@dataclass
class KVCache:
    """Device tensors of the paged cache: k, v [num_blocks][Hkv][16][D]; block_tables [B][max_blocks] int32."""
    k: torch.Tensor
    v: torch.Tensor
    block_tables: torch.Tensor
    num_q_heads: int

    def struct(self) -> aspd_kv:
        nb, hkv, bs, d = self.k.shape
        return aspd_kv(_ptr(self.k), _ptr(self.v), _ptr(self.block_tables), nb, bs, self.num_q_heads, hkv, d,
                       self.block_tables.shape[1], _DTYPE[self.k.dtype])


class BatchState:
    """Caller-owned decode state of a batch (device int arrays), see aspd_state in aspd.h."""

    def __init__(self, B: int, owner_stride: int, device):
        self.B = B
        self.NB = 0
        self.device = device
        self.stage_base = torch.zeros(B, dtype=torch.int32, device=device)
        self.seq_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.cu_branches = None
        self.branch_len = None
        self.owner_stride = int(owner_stride)
        self.slot_owner = torch.zeros(B, self.owner_stride, dtype=torch.uint8, device=device)
        self.fault = torch.zeros(1, dtype=torch.int32, device=device)
        self.main_pos = torch.zeros(B, dtype=torch.int32, device=device)
        self.stage_open = torch.zeros(B, dtype=torch.int32, device=device)
        self.pos_mode = POS_SAME_SEQ   # the position paradigm every metadata call on this state uses

    def open_parallel(self, cu_branches: torch.Tensor) -> None:
        """New parallel stage: branch layout given by the caller, branch lengths start at zero."""
        self.cu_branches = cu_branches.to(device=self.device, dtype=torch.int32)
        self.NB = int(cu_branches[-1])
        self.branch_len = torch.zeros(max(self.NB, 1), dtype=torch.int32, device=self.device)
        # the caller opens the stage, so the caller marks it (see aspd_state.stage_open_d)
        self.stage_open.copy_((self.cu_branches[1:] > self.cu_branches[:-1]).to(torch.int32))

    def struct(self) -> aspd_state:
        return aspd_state(self.B, self.NB, _ptr(self.stage_base), _ptr(self.seq_len), _ptr(self.cu_branches),
                          _ptr(self.branch_len), _ptr(self.slot_owner), self.owner_stride, _ptr(self.fault),
                          _ptr(self.main_pos), _ptr(self.stage_open))


class Step:
    """Outputs of one aspd_build_branch_meta call (device arrays sized for NQ rows)."""

    def __init__(self, NQ: int, n_cu: int, B: int, device, max_new_per_seq: int = 0, max_workgroups: int = 0):
        self.NQ = int(NQ)
        self.max_new_per_seq = int(max_new_per_seq)   # tuning hint, 0 = unknown
        self.max_workgroups = int(max_workgroups)     # cap of the attention grids, 0 = none
        self.shared_mask = 0                          # 1: the ablation's shared mask (see aspd_step.shared_mask)
        self.plan = None                              # device buffer for the step's plan (see aspd_step.plan_d)
        self.plan_key = 0                             # as aspd_build_branch_meta left it
        i32 = dict(dtype=torch.int32, device=device)
        n = max(self.NQ, 1)
        self.cu_new = torch.zeros(n_cu + 1, **i32)
        self.cu_seq_new = torch.zeros(B + 1, **i32)
        self.q_seq = torch.zeros(n, **i32)
        self.q_branch = torch.zeros(n, **i32)
        self.position_ids = torch.zeros(n, **i32)
        self.logical_slot = torch.zeros(n, **i32)
        self.slot_mapping = torch.zeros(n, dtype=torch.int64, device=device)
        self.kv_len = torch.zeros(n, **i32)

    def struct(self) -> aspd_step:
        plan_bytes = 0 if self.plan is None else self.plan.numel() * self.plan.element_size()
        return aspd_step(self.NQ, self.max_new_per_seq, self.max_workgroups, self.shared_mask, _ptr(self.cu_new),
                         _ptr(self.cu_seq_new),
                         _ptr(self.q_seq), _ptr(self.q_branch), _ptr(self.position_ids), _ptr(self.logical_slot),
                         _ptr(self.slot_mapping), _ptr(self.kv_len), _ptr(self.plan), plan_bytes, self.plan_key)


def aspd_build_branch_meta(kv: KVCache, state: BatchState, stage: int, new_len: torch.Tensor | None,
                           NQ: int = 0, step: Step | None = None, stream=None,
                           max_new_per_seq: int = 0, max_workgroups: int = 0, plan: bool = True) -> Step | None:
    """See aspd.h.  `NQ` = sum of new_len, known to the caller.  Returns the Step (None for MERGE,
    where new_len, if given, says per sequence whether its stage ends).  `plan`: give the step a plan
    buffer (allocated here on the step's first use) so that the attention calls start from the plan."""
    kvs, sts = kv.struct(), state.struct()
    if stage == STAGE_MERGE:
        rc = lib().aspd_build_branch_meta(C.byref(kvs), C.byref(sts), stage, state.pos_mode, _ptr(new_len), None,
                                          _stream(stream))
        if rc != OK:
            raise AspdError(rc, "aspd_build_branch_meta")
        return None
    if step is None:
        step = Step(NQ, state.B if stage == STAGE_SERIAL else state.NB, state.B, state.device,
                    max_new_per_seq, max_workgroups)
    if plan and step.plan is None and step.NQ > 0:
        step.plan = torch.empty(aspd_plan_bytes(kv, state.B, step.NQ), dtype=torch.uint8, device=state.device)
    sps = step.struct()
    rc = lib().aspd_build_branch_meta(C.byref(kvs), C.byref(sts), stage, state.pos_mode, _ptr(new_len),
                                      C.byref(sps), _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_build_branch_meta")
    step.plan_key = int(sps.plan_key)   # the one host field the library writes
    return step


def aspd_renumber_branches(state: BatchState, new_cu_branches: torch.Tensor, stream=None) -> None:
    """See aspd.h: switches `state` to the branch numbering `new_cu_branches` ([B+1], any device);
    branches of stages still running keep their lengths, the others start at zero."""
    new_cu = new_cu_branches.to(device=state.device, dtype=torch.int32)
    new_nb = int(new_cu_branches[-1])
    new_len = torch.zeros(max(new_nb, 1), dtype=torch.int32, device=state.device)
    if state.cu_branches is None:          # no branch has ever been open: nothing to carry over
        state.cu_branches, state.branch_len, state.NB = new_cu, new_len, new_nb
        state.stage_open.copy_((new_cu[1:] > new_cu[:-1]).to(torch.int32))
        return
    sts = state.struct()
    rc = lib().aspd_renumber_branches(C.byref(sts), _ptr(new_cu), _ptr(new_len), _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_renumber_branches")
    state.cu_branches, state.branch_len, state.NB = new_cu, new_len, new_nb


def aspd_rope_append(kv: KVCache, step: Step, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                     rope_theta: float, stream=None) -> torch.Tensor:
    """See aspd.h: rotates q in place, writes rotated k_new and plain v_new into the cache.  Returns q."""
    kvs, sps = kv.struct(), step.struct()
    rc = lib().aspd_rope_append(C.byref(kvs), C.byref(sps), _ptr(q), _ptr(k_new), _ptr(v_new),
                                C.c_float(rope_theta), _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_rope_append")
    return q


def aspd_workspace_bytes(kv: KVCache, B: int, NQ: int) -> int:
    kvs = kv.struct()
    return int(lib().aspd_workspace_bytes(C.byref(kvs), B, NQ))


def aspd_plan_bytes(kv: KVCache, B: int, NQ: int) -> int:
    kvs = kv.struct()
    return int(lib().aspd_plan_bytes(C.byref(kvs), B, NQ))


def _attn(name, kv, state, step, q, out, lse, sm_scale, workspace, stream):
    kvs, sts, sps = kv.struct(), state.struct(), step.struct()
    if out is None:
        out = torch.empty_like(q)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = getattr(lib(), name)(C.byref(kvs), C.byref(sts), C.byref(sps), _ptr(q), _ptr(out), _ptr(lse),
                              C.c_float(sm_scale), _ptr(workspace), nbytes, _stream(stream))
    if rc != OK:
        raise AspdError(rc, name)
    return out


def aspd_attn_parallel_decode(kv, state, step, q, workspace, out=None, lse=None, sm_scale=0.0, stream=None):
    return _attn("aspd_attn_parallel_decode", kv, state, step, q, out, lse, sm_scale, workspace, stream)


def aspd_attn_branch_chunk(kv, state, step, q, workspace, out=None, lse=None, sm_scale=0.0, stream=None):
    return _attn("aspd_attn_branch_chunk", kv, state, step, q, out, lse, sm_scale, workspace, stream)


def aspd_attn_serial_decode(kv, state, step, q, workspace, out=None, lse=None, sm_scale=0.0, stream=None):
    return _attn("aspd_attn_serial_decode", kv, state, step, q, out, lse, sm_scale, workspace, stream)


def aspd_sequence_plan_bytes(kv: KVCache, B: int, NQ: int) -> int:
    kvs = kv.struct()
    return int(lib().aspd_sequence_plan_bytes(C.byref(kvs), B, NQ))


def aspd_build_sequence_meta(kv: KVCache, state: BatchState, cu_runs: torch.Tensor, run_branch: torch.Tensor,
                             run_len: torch.Tensor, NQ: int, step: Step | None = None, stream=None,
                             max_workgroups: int = 0) -> Step:
    """See aspd.h: the metadata of every token of a batch of whole multi-stage sequences.  The three int32
    device arrays describe the layout; `NQ` = sum of run_len, known to the caller."""
    kvs, sts = kv.struct(), state.struct()
    if step is None:
        step = Step(NQ, 0, state.B, state.device, 0, max_workgroups)
    need = aspd_sequence_plan_bytes(kv, state.B, step.NQ)
    if step.plan is None or step.plan.numel() < need:
        step.plan = torch.empty(max(need, 256), dtype=torch.uint8, device=state.device)
    lay = aspd_layout(int(run_branch.numel()), _ptr(cu_runs), _ptr(run_branch), _ptr(run_len))
    sps = step.struct()
    rc = lib().aspd_build_sequence_meta(C.byref(kvs), C.byref(sts), C.byref(lay), state.pos_mode, C.byref(sps),
                                        _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_build_sequence_meta")
    step.plan_key = int(sps.plan_key)
    return step


def aspd_attn_full_sequence(kv, state, step, q, workspace, out=None, lse=None, sm_scale=0.0, stream=None):
    return _attn("aspd_attn_full_sequence", kv, state, step, q, out, lse, sm_scale, workspace, stream)


def aspd_attn_parallel_decode_static(kv, state, step, q, out, lse=None, sm_scale=0.0, stream=None):
    """See aspd.h: parallel decode on the library's own static scratch.  `out` is the caller's (nothing is
    allocated here either)."""
    kvs, sts, sps = kv.struct(), state.struct(), step.struct()
    rc = lib().aspd_attn_parallel_decode_static(C.byref(kvs), C.byref(sts), C.byref(sps), _ptr(q), _ptr(out), _ptr(lse),
                                                C.c_float(sm_scale), _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_attn_parallel_decode_static")
    return out


def aspd_workspace_init(workspace: torch.Tensor, stream=None) -> None:
    rc = lib().aspd_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_workspace_init")


def aspd_probe_read_bandwidth(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    rc = lib().aspd_probe_read_bandwidth(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream))
    if rc != OK:
        raise AspdError(rc, "aspd_probe_read_bandwidth")


def new_workspace(kv: KVCache, B: int, NQ: int) -> torch.Tensor:
    """Device scratch of the size the attention calls ask for (256-byte aligned by the allocator),
    prepared with aspd_workspace_init."""
    ws = torch.empty(aspd_workspace_bytes(kv, B, NQ), dtype=torch.uint8, device=kv.k.device)
    aspd_workspace_init(ws)
    return ws
