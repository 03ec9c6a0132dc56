"""Test helper: drive the GPU library (through the Python binding of the C ABI) along the same
append history the oracle replays.  Only the binding and the input generators are used here."""
import numpy as np
import torch

import aspd_workloads as W
from paper_2508_08895_amd import binding as A


class GpuBatch:
    def __init__(self, wl, device="cuda", poison_unmapped=True):
        self.wl = wl
        self.dev = torch.device(device)
        k, v = wl.k_cache, wl.v_cache
        if poison_unmapped:
            # blocks no table refers to hold NaN: any read outside the block tables shows up
            used = np.unique(wl.block_tables[wl.block_tables >= 0])
            free = np.setdiff1d(np.arange(wl.num_blocks), used)
            if free.size:
                k, v = k.clone(), v.clone()
                k[torch.from_numpy(free)] = float("nan")
                v[torch.from_numpy(free)] = float("nan")
        self.kv = A.KVCache(k.to(self.dev), v.to(self.dev),
                            torch.from_numpy(wl.block_tables).to(self.dev), wl.num_q_heads)
        self.state = A.BatchState(wl.B, wl.max_blocks_per_seq * wl.block_size, self.dev)
        # for any step this batch can take: no call brings more rows than the block tables hold tokens
        self.workspace = A.new_workspace(self.kv, wl.B, int((wl.block_tables >= 0).sum()) * wl.block_size)

    def _dev_i32(self, x):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(self.dev)

    def serial(self, new_len):
        return A.aspd_build_branch_meta(self.kv, self.state, A.STAGE_SERIAL, self._dev_i32(new_len),
                                        NQ=int(np.sum(new_len)))

    def open_parallel(self):
        self.state.open_parallel(torch.from_numpy(self.wl.cu_branches))

    def parallel(self, new_len):
        return A.aspd_build_branch_meta(self.kv, self.state, A.STAGE_PARALLEL, self._dev_i32(new_len),
                                        NQ=int(np.sum(new_len)))

    def merge(self, which=None):
        A.aspd_build_branch_meta(self.kv, self.state, A.STAGE_MERGE,
                                 None if which is None else self._dev_i32(np.asarray(which, dtype=np.int32)))

    def renumber(self, num_branches):
        """Branch count per sequence after some stages opened / ended."""
        cu = np.zeros(len(num_branches) + 1, dtype=np.int32)
        np.cumsum(num_branches, out=cu[1:])
        A.aspd_renumber_branches(self.state, torch.from_numpy(cu))

    def mixed(self, new_len_branch, new_len_main):
        both = np.concatenate([np.asarray(new_len_branch, dtype=np.int32), np.asarray(new_len_main, dtype=np.int32)])
        return A.aspd_build_branch_meta(self.kv, self.state, A.STAGE_MIXED, self._dev_i32(both), NQ=int(both.sum()))

    def grow_to(self, branch_len):
        """Prefix, open the parallel stage, grow the branches one token per active branch per step."""
        self.serial(self.wl.prefix_len)
        self.open_parallel()
        last = None
        for new_len in W.interleaved_history(branch_len):
            last = self.parallel(new_len)
        return last

    def fault(self) -> int:
        return int(self.state.fault.item())


STEP_FIELDS = ("cu_new", "cu_seq_new", "q_seq", "q_branch", "position_ids", "logical_slot", "slot_mapping",
               "kv_len")


def assert_step_equal(step, meta):
    """GPU Step vs oracle StepMeta, bit-exact."""
    assert step.NQ == meta.NQ
    for f in STEP_FIELDS:
        got = getattr(step, f).cpu().numpy()
        want = getattr(meta, f)
        if f not in ("cu_new", "cu_seq_new"):
            got = got[:meta.NQ]
        assert got.dtype == want.dtype, f
        assert np.array_equal(got, want), (f, got[:16], want[:16])


def assert_state_equal(gb, tt):
    st = gb.state
    T = tt.seq_len()
    L = tt.stage_base()
    assert np.array_equal(st.seq_len.cpu().numpy(), T)
    assert np.array_equal(st.stage_base.cpu().numpy(), L)
    bl = tt.branch_len()
    if bl.size:
        assert np.array_equal(st.branch_len.cpu().numpy()[:bl.size], bl)
    own_g = st.slot_owner.cpu().numpy()
    own_o = tt.slot_owner(st.owner_stride)
    for s in range(gb.wl.B):
        assert np.array_equal(own_g[s, L[s]:T[s]], own_o[s, L[s]:T[s]]), s
    assert st.stage_open.cpu().numpy().astype(bool).tolist() == [bool(x) for x in tt.cur_parallel]
    assert gb.fault() == 0
