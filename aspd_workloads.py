"""Seeded synthetic inputs for branch-isolated attention over a paged KV cache.

This module only draws shapes and random tensors.  It contains none of the
method's arithmetic: no position ids, no slot assignment, no mask, no
attention.  Both the CPU oracle's tests and the GPU library's tests feed on
the arrays produced here; neither side's code is imported.

Workload shapes follow the paper's parallel-stage statistics: a handful of
branches per parallel stage (Table 2 and Table 5 report 2.4 to 3.2 branches on
average), branches of a few tens of tokens (Sec. 4.5.3 finds the best fixed
interval at 32, the average branch length), and serial contexts of up to 8k to
12k tokens (Sec. 4.1, Sec. 4.4).  The five named configurations bracket those
figures.  They stand in for the paper's evaluation sets, whose items are not
used: only lengths, counts and value distributions matter to attention.

Draw order (numpy PCG64, seed = SEED_BASE + configuration index), fixed so that
every consumer sees the same arrays:
  1. per-sequence serial-prefix length  L_s
  2. per-sequence branch count          K_s
  3. per-branch length                  n_b
  4. block-table placement (one permutation of the pool)
  5. K cache, 6. V cache  (whole pool, iid normal * sigma, rounded to dtype)
  7. queries, on demand, in call order
Integer ranges are inclusive.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

SEED_BASE = 250808895
BLOCK_SIZE = 16

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclass
class Workload:
    """One batch of sequences sharing a paged KV pool (all arrays on the CPU)."""

    name: str
    dtype: str                    # "f32" | "bf16"
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    sigma: float
    prefix_len: np.ndarray        # [B]  int32, serial-prefix tokens per sequence
    num_branches: np.ndarray      # [B]  int32
    branch_len: np.ndarray        # [NB] int32, tokens per branch (see each config for what they count)
    block_tables: np.ndarray      # [B][max_blocks_per_seq] int32, -1 = not allocated
    num_blocks: int
    k_cache: torch.Tensor         # [num_blocks][Hkv][block_size][D]
    v_cache: torch.Tensor         # same
    rng: np.random.Generator = field(repr=False, default=None)
    extra_tokens_per_branch: int = 0   # capacity reserved beyond branch_len, per branch
    extra_tokens_per_seq: int = 0      # capacity reserved for serial tokens after the merge

    @property
    def B(self) -> int:
        return int(self.prefix_len.shape[0])

    @property
    def NB(self) -> int:
        return int(self.branch_len.shape[0])

    @property
    def cu_branches(self) -> np.ndarray:
        cu = np.zeros(self.B + 1, dtype=np.int32)
        np.cumsum(self.num_branches, out=cu[1:])
        return cu

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def torch_dtype(self) -> torch.dtype:
        return _TORCH_DTYPE[self.dtype]

    def draw_q(self, num_rows: int) -> torch.Tensor:
        """Next query batch [num_rows][Hq][D] in the workload's dtype."""
        return _normal(self.rng, (num_rows, self.num_q_heads, self.head_dim), self.sigma, self.torch_dtype)


def _normal(rng: np.random.Generator, shape, sigma: float, dtype: torch.dtype) -> torch.Tensor:
    """iid N(0, sigma^2) drawn in float32, then rounded to dtype (nearest-even).

    Drawn in bounded pieces so that a multi-gigabyte pool never needs a second
    full-size float32 copy.
    """
    total = int(np.prod(shape))
    out = torch.empty(total, dtype=dtype)
    piece = 1 << 24
    for lo in range(0, total, piece):
        hi = min(total, lo + piece)
        x = rng.standard_normal(hi - lo, dtype=np.float32)
        x *= np.float32(sigma)
        out[lo:hi] = torch.from_numpy(x).to(dtype)
    return out.reshape(shape)


def make_workload(name: str, seed: int, *, dtype: str, num_q_heads: int, num_kv_heads: int, head_dim: int,
                  sigma: float, prefix_range, branches_range, branch_len_range, batch: int,
                  pool_factor: float, extra_tokens_per_branch: int, extra_tokens_per_seq: int,
                  identity_tables: bool = False, prefix_len=None, num_branches=None,
                  branch_len=None) -> Workload:
    """Draw one workload.  Explicit prefix_len/num_branches/branch_len override the draws
    (the corresponding draw is then skipped, later draws keep their order)."""
    rng = np.random.default_rng(seed)
    B = batch
    if prefix_len is None:
        prefix_len = rng.integers(prefix_range[0], prefix_range[1], size=B, endpoint=True)
    prefix_len = np.asarray(prefix_len, dtype=np.int32)
    if num_branches is None:
        num_branches = rng.integers(branches_range[0], branches_range[1], size=B, endpoint=True)
    num_branches = np.asarray(num_branches, dtype=np.int32)
    NB = int(num_branches.sum())
    if branch_len is None:
        branch_len = rng.integers(branch_len_range[0], branch_len_range[1], size=NB, endpoint=True)
    branch_len = np.asarray(branch_len, dtype=np.int32)
    assert prefix_len.shape == (B,) and num_branches.shape == (B,) and branch_len.shape == (NB,)

    # capacity (tokens) each sequence may ever hold in this workload
    cu = np.concatenate([[0], np.cumsum(num_branches)])
    cap_tokens = np.empty(B, dtype=np.int64)
    for s in range(B):
        nb = branch_len[cu[s]:cu[s + 1]].astype(np.int64)
        cap_tokens[s] = int(prefix_len[s]) + int(nb.sum()) + int(num_branches[s]) * extra_tokens_per_branch \
            + extra_tokens_per_seq
    cap_blocks = (cap_tokens + BLOCK_SIZE - 1) // BLOCK_SIZE
    need = int(cap_blocks.sum())
    max_blocks = int(cap_blocks.max())
    num_blocks = need if identity_tables else int(np.ceil(need * pool_factor))

    block_tables = np.full((B, max_blocks), -1, dtype=np.int32)
    if identity_tables:
        order = np.arange(num_blocks, dtype=np.int64)
    else:
        order = rng.permutation(num_blocks)
    at = 0
    for s in range(B):
        c = int(cap_blocks[s])
        block_tables[s, :c] = order[at:at + c]
        at += c

    tdt = _TORCH_DTYPE[dtype]
    shape = (num_blocks, num_kv_heads, BLOCK_SIZE, head_dim)
    k_cache = _normal(rng, shape, sigma, tdt)
    v_cache = _normal(rng, shape, sigma, tdt)
    return Workload(name=name, dtype=dtype, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                    head_dim=head_dim, block_size=BLOCK_SIZE, sigma=sigma, prefix_len=prefix_len,
                    num_branches=num_branches, branch_len=branch_len, block_tables=block_tables,
                    num_blocks=num_blocks, k_cache=k_cache, v_cache=v_cache, rng=rng,
                    extra_tokens_per_branch=extra_tokens_per_branch,
                    extra_tokens_per_seq=extra_tokens_per_seq)


# ----------------------------------------------------------------------------------------------
# The five named configurations.  `branch_len` counts, for configs 1-4, the tokens of a branch
# INCLUDING the one the measured parallel-decode step appends; for config 5 it counts the tokens
# present BEFORE the 16-token chunk pass (the chunk takes n -> n+16, the decode step -> n+17).
# ----------------------------------------------------------------------------------------------
_LLM7B = dict(dtype="bf16", num_q_heads=32, num_kv_heads=8, head_dim=128, sigma=0.5)


def config(index: int, *, scale: float = 1.0, batch: int | None = None) -> Workload:
    """Configuration `index` in 1..5.  `scale` < 1 shrinks prefix lengths (and `batch` the
    batch) for quick tests of the same structure; the defaults are the full sizes."""
    seed = SEED_BASE + index

    def sc(x):
        return max(1, int(round(x * scale)))

    if index == 1:
        return make_workload("cfg1_tiny_f32", seed, dtype="f32", num_q_heads=4, num_kv_heads=4, head_dim=64,
                             sigma=1.0, prefix_range=None, branches_range=None, branch_len_range=None,
                             batch=1, pool_factor=1.0, extra_tokens_per_branch=0, extra_tokens_per_seq=2,
                             identity_tables=True, prefix_len=[64], num_branches=[3], branch_len=[5, 9, 16])
    if index == 2:
        return make_workload("cfg2_7b_b1", seed, **_LLM7B, prefix_range=None, branches_range=None,
                             branch_len_range=None, batch=1, pool_factor=4.0, extra_tokens_per_branch=0,
                             extra_tokens_per_seq=0, prefix_len=[sc(2048)], num_branches=[4],
                             branch_len=[64, 64, 64, 64])
    if index == 3:
        return make_workload("cfg3_b16_mixed", seed, **_LLM7B, prefix_range=(sc(512), sc(4096)),
                             branches_range=(2, 8), branch_len_range=(16, 256), batch=batch or 16,
                             pool_factor=1.5, extra_tokens_per_branch=0, extra_tokens_per_seq=0)
    if index == 4:
        b = batch or 4
        return make_workload("cfg4_long_prefix", seed, **_LLM7B, prefix_range=None, branches_range=None,
                             branch_len_range=(32, 192), batch=b, pool_factor=1.25,
                             extra_tokens_per_branch=0, extra_tokens_per_seq=32,
                             prefix_len=[sc(16384)] * b, num_branches=[6] * b)
    if index == 5:
        return make_workload("cfg5_b64_chunk", seed, **_LLM7B, prefix_range=(sc(1024), sc(8192)),
                             branches_range=(2, 10), branch_len_range=(8, 128), batch=batch or 64,
                             pool_factor=1.1, extra_tokens_per_branch=17, extra_tokens_per_seq=8)
    raise ValueError(f"no configuration {index}")


def random_small(seed: int, *, dtype: str = "bf16", num_q_heads: int = 32, num_kv_heads: int = 8,
                 head_dim: int = 128, batch: int = 3, prefix_range=(0, 70), branches_range=(1, 5),
                 branch_len_range=(1, 40), extra_tokens_per_branch: int = 20,
                 extra_tokens_per_seq: int = 4, sigma: float | None = None) -> Workload:
    """Small ragged workloads for randomized parity cases (several pages and a ragged tail)."""
    if sigma is None:
        sigma = 1.0 if dtype == "f32" else 0.5
    return make_workload(f"small_{seed}", seed, dtype=dtype, num_q_heads=num_q_heads,
                         num_kv_heads=num_kv_heads, head_dim=head_dim, sigma=sigma,
                         prefix_range=prefix_range, branches_range=branches_range,
                         branch_len_range=branch_len_range, batch=batch, pool_factor=2.0,
                         extra_tokens_per_branch=extra_tokens_per_branch,
                         extra_tokens_per_seq=extra_tokens_per_seq)


def interleaved_history(target_len) -> list:
    """Append history that grows every branch from empty to target_len[b] tokens with all
    branches starting together: step t appends one token to every branch with target_len[b] > t
    (the inference-time arrangement, one token per active branch per step).  Returns the list of
    per-step new_len arrays (int32 [NB], entries 0 or 1)."""
    target_len = np.asarray(target_len, dtype=np.int32)
    steps = int(target_len.max()) if target_len.size else 0
    return [(target_len > t).astype(np.int32) for t in range(steps)]


def random_layouts(wl: Workload, seed: int, max_stages: int = 3, max_branches: int = 6, fill: float = 1.0) -> list:
    """Per sequence of `wl` the runs of a whole multi-stage sequence in cache order, [(branch, tokens)]:
    (0, n) main-branch tokens, (k, n) the k-th branch of a parallel stage (branches of a stage numbered
    1..K in order); serial and parallel stages alternate, a sequence may start or end with either, runs
    may be empty.  The tokens of a sequence fill `fill` of what its block table has room for."""
    rng = np.random.default_rng(seed)
    out = []
    for s in range(wl.B):
        room = int(fill * wl.block_size * int((wl.block_tables[s] >= 0).sum()))
        P = int(rng.integers(0, max_stages + 1))
        w = rng.random(2 * P + 1) + 0.05
        if P > 0 and rng.random() < 0.25:
            w[0] = 0.0                       # the sequence starts with a parallel stage
        if P > 0 and rng.random() < 0.25:
            w[-1] = 0.0                      # ... or ends with one
        seg = np.floor(room * w / w.sum()).astype(np.int64)
        runs = []
        for i, n in enumerate(seg):
            if i % 2 == 0:
                runs.append((0, int(n)))
            else:
                K = int(rng.integers(1, max_branches + 1))
                cut = np.sort(rng.integers(0, int(n) + 1, size=K - 1))
                lens = np.diff(np.concatenate([[0], cut, [int(n)]]))
                runs.extend((k + 1, int(lens[k])) for k in range(K))
        out.append(runs)
    return out
