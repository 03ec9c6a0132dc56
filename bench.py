#!/usr/bin/env python3
"""Benchmark of the ASPD attention hot path on one MI355X.

Metric (one attention layer): branch-query tokens per second of the parallel-decode call, with the HBM
bandwidth it achieves against the 8 TB/s peak.  The default run measures it on all five named
configurations (`per_config`); the headline `value` is the figure of configuration 5, the largest.

A step is one pass of the whole hot path over configuration 5's batch, per attention layer: the
16-token branch-chunk fill that opens a parallel stage (metadata + attention), one parallel-decode step
(metadata + attention), the merge (metadata only) and the serial-decode steps that follow (metadata +
attention each), all through the C ABI of libaspd.so on one HIP stream, captured in a HIP graph.  Inputs
(KV pools, block tables, queries) are resident in HBM before the timed region; the decode state is
restored from a snapshot at the start of every step (small device copies inside the timed region), so
that every step does identical work.  `ms_per_step` is that step, timed over `--steps` steps.

Per call kind the average launch is measured separately: REP back-to-back launches of the one attention
kernel (no metadata calls between them), captured once, timed with events on the launch stream, each
launch on another KV pool so that no timed byte comes from a cache.  `roofline` is the parallel-decode
kernel on configuration 5 alone against the HBM peak; `roofline_chunk` the branch-chunk kernel against the
dense bf16 MFMA peak; `cpu_baseline` the CPU oracle (its C writing, OpenMP on all host cores) on a bounded sample.
One GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
MFMA_BF16_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak

# name -> configuration index, chunk tokens per branch (0: no chunk call), serial steps after the merge,
#         tokens every branch holds before the step relative to the configuration's branch_len
WORKLOADS = {
    "cfg1": dict(index=1, chunk=0, serial=1, base_offset=-1,
                 what="config 1 (B=1, 4q/4kv/64 fp32, prefix 64, branches 5/9/16, contiguous KV): "
                      "parallel-decode step, merge, one serial-decode step"),
    "cfg2": dict(index=2, chunk=0, serial=0, base_offset=-1,
                 what="config 2 (B=1, 32q/8kv/128 bf16, prefix 2048, 4 branches at 64, paged 16): one parallel-decode step"),
    "cfg3": dict(index=3, chunk=0, serial=0, base_offset=-1,
                 what="config 3 (B=16 mixed, prefix 512..4096, 2..8 branches of 16..256): one parallel-decode step"),
    "cfg4": dict(index=4, chunk=0, serial=32, base_offset=-1,
                 what="config 4 (B=4, prefix 16384, 6 branches of 32..192): parallel-decode step, merge, "
                      "32 serial-decode steps"),
    "cfg5": dict(index=5, chunk=16, serial=4, base_offset=0,
                 what="config 5 (B=64, prefix 1024..8192, 2..10 branches of 8..128, paged 16): 16-token branch chunk, "
                      "parallel-decode step, merge, 4 serial-decode steps"),
    "cycle4": dict(index=4, chunk=16, serial=32, base_offset=-17,
                   what="config 4's batch (B=4, prefix 16384, 6 branches of 32..192): 16-token branch chunk, parallel-decode step, "
                        "merge, 32 serial-decode steps"),
}
DEFAULT_SET = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")
HEADLINE = "cfg5"


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def measure(name, args, timed, mods):
    """Everything about one workload: per-call launch times (always) and the timed step (`timed`)."""
    np, torch, W, A = mods
    dev = torch.device("cuda:0")
    spec = WORKLOADS[name]
    t0 = time.time()
    wl = W.config(spec["index"])
    log(f"{name}: generated in {time.time() - t0:.1f}s")

    bt_dev = torch.from_numpy(wl.block_tables).to(dev)
    kv = A.KVCache(wl.k_cache.to(dev), wl.v_cache.to(dev), bt_dev, wl.num_q_heads)
    state = A.BatchState(wl.B, wl.max_blocks_per_seq * 16, dev)
    B, NB = wl.B, wl.NB
    # Distinct KV pools ("layers", as a model has one cache per layer) that consecutive attention calls
    # rotate through, so that no call finds its pages in the 256 MB memory-side cache from the call
    # before: every timed byte comes from HBM.  Layer 0 is the seeded pool; the others hold values
    # of the same distribution drawn on the device.  (Configurations 1 and 2 are smaller than the caches
    # however many pools there are: their launches are bound by latency, see latency_aware_bound_us.)
    elt = 2 if wl.dtype == "bf16" else 4
    active = int(wl.prefix_len.sum() + wl.branch_len.sum()) * 2 * wl.num_kv_heads * wl.head_dim * elt
    n_layers = args.layers or int(min(32, max(2, -(-int(1.5e9) // active))))
    kvs = [kv]
    for _ in range(n_layers - 1):
        k2 = (torch.randn(wl.k_cache.shape, device=dev, dtype=torch.float32) * wl.sigma).to(wl.torch_dtype)
        v2 = (torch.randn(wl.v_cache.shape, device=dev, dtype=torch.float32) * wl.sigma).to(wl.torch_dtype)
        kvs.append(A.KVCache(k2, v2, bt_dev, wl.num_q_heads))
    log(f"{name}: {n_layers} KV pools of {2 * wl.k_cache.numel() * elt / 1e6:.0f} MB, {active / 1e6:.1f} MB read per call")
    rot = [0]

    def next_kv():
        rot[0] = (rot[0] + 1) % n_layers
        return kvs[rot[0]]

    base_len = wl.branch_len + spec["base_offset"]
    assert (base_len >= 0).all()

    def dev_i32(x):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)

    # ---- bring the cache state to the start of a step (untimed)
    A.aspd_build_branch_meta(kv, state, A.STAGE_SERIAL, dev_i32(wl.prefix_len), NQ=int(wl.prefix_len.sum()), plan=False)
    state.open_parallel(torch.from_numpy(wl.cu_branches))
    for new_len in W.interleaved_history(base_len):
        A.aspd_build_branch_meta(kv, state, A.STAGE_PARALLEL, dev_i32(new_len), NQ=int(new_len.sum()), plan=False)
    torch.cuda.synchronize()
    assert int(state.fault.item()) == 0
    live = (state.stage_base, state.seq_len, state.branch_len, state.slot_owner, state.stage_open)
    snap = [t.clone() for t in live]

    # ---- pre-allocated per-call inputs and outputs
    C, S = spec["chunk"], spec["serial"]
    g = torch.Generator().manual_seed(W.SEED_BASE)

    def rand_q(n):
        return (torch.randn(n, wl.num_q_heads, wl.head_dim, generator=g) * wl.sigma).to(wl.torch_dtype).to(dev)

    ws = A.new_workspace(kv, B, max(C * NB, NB, B))
    kmax = int(wl.num_branches.max())
    calls = []  # (kind, stage, new_len_d, step, q, fn)
    if C:
        calls.append(("chunk", A.STAGE_PARALLEL, dev_i32(np.full(NB, C)), A.Step(C * NB, NB, B, dev, max_new_per_seq=C * kmax),
                      rand_q(C * NB), A.aspd_attn_branch_chunk))
    calls.append(("parallel", A.STAGE_PARALLEL, dev_i32(np.ones(NB)), A.Step(NB, NB, B, dev, max_new_per_seq=kmax), rand_q(NB),
                  A.aspd_attn_parallel_decode))
    if S:
        calls.append(("merge", A.STAGE_MERGE, None, None, None, None))
        ones_b = dev_i32(np.ones(B))
        for _ in range(S):
            calls.append(("serial", A.STAGE_SERIAL, ones_b, A.Step(B, B, B, dev, max_new_per_seq=1), rand_q(B),
                          A.aspd_attn_serial_decode))
    outs = {id(c): (torch.empty_like(c[4]) if c[4] is not None else None) for c in calls}
    n_attn = sum(1 for c in calls if c[5] is not None)
    ROUND = -(-n_layers // n_attn)   # steps after which every pool has been read once

    def one_step(snaps=None, offset=0):
        rot[0] = (offset * n_attn) % n_layers
        for dst, src in zip(live, snap):
            dst.copy_(src)
        for c in calls:
            kind, stage, new_len, step, q, fn = c
            A.aspd_build_branch_meta(kv, state, stage, new_len, step=step)
            if fn is None:
                continue
            if snaps is not None and kind not in snaps:   # state as the first call of this kind sees it
                snaps[kind] = ([t.clone() for t in live], c)
            fn(next_kv(), state, step, q, ws, out=outs[id(c)])

    # ---- algorithmic bytes (unique visible KV + Q and O + tables + tags) and, for the chunk, flops
    kv_tok_bytes = 2 * wl.num_kv_heads * wl.head_dim * elt
    cu = wl.cu_branches
    per_seq_branch_tokens = np.add.reduceat(base_len, cu[:-1]).astype(np.int64)
    T = wl.prefix_len.astype(np.int64) + per_seq_branch_tokens
    bytes_of, tokens_of = {}, {}
    Tn = T.copy()
    chunk_flops = 0
    for c in calls:
        kind = c[0]
        if kind == "merge":
            continue
        if kind == "chunk":
            Tn = Tn + C * wl.num_branches
            nq = C * NB
            # token j of a branch that held n tokens attends prefix + n + j + 1 keys: 4 * D flops per key and head
            seq_of = np.repeat(np.arange(B), wl.num_branches)
            keys = (wl.prefix_len[seq_of].astype(np.int64) + base_len) * C + C * (C + 1) // 2
            chunk_flops = int(keys.sum()) * 4 * wl.head_dim * wl.num_q_heads
        elif kind == "parallel":
            Tn = Tn + wl.num_branches
            nq = NB
        else:
            Tn = Tn + 1
            nq = B
        b = int(Tn.sum()) * kv_tok_bytes + 2 * nq * wl.num_q_heads * wl.head_dim * elt \
            + 4 * int(((Tn + 15) // 16).sum()) + (0 if kind == "serial" else int((Tn - wl.prefix_len).sum()))
        bytes_of.setdefault(kind, []).append(b)
        tokens_of.setdefault(kind, []).append(nq)

    # ---- the step as a HIP graph (every call only enqueues kernels on the current stream, so the
    # whole step is capturable); replay must reproduce the eager outputs
    snaps = {}
    one_step(snaps)
    torch.cuda.synchronize()
    assert int(state.fault.item()) == 0
    eager_out = {k: v.clone() for k, v in outs.items() if v is not None}
    graphs = []
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_step()
        torch.cuda.current_stream().wait_stream(side)
        for r in range(ROUND if timed else 1):          # one captured step per rotation offset
            g_r = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_r):
                one_step(offset=r)
            graphs.append(g_r)
        for v in outs.values():
            if v is not None:
                v.zero_()
        graphs[0].replay()
        torch.cuda.synchronize()
        tol = 2e-2 if wl.dtype == "bf16" else 1e-5
        for k, v in eager_out.items():
            # pairs of pages are handed to waves dynamically, so the summation order (not the math) may differ
            assert torch.allclose(outs[k].float(), v.float(), atol=tol, rtol=0), "graph replay differs from the eager step"

    def run_step(t):
        if graphs:
            graphs[t % len(graphs)].replay()
        else:
            one_step(offset=t % ROUND)

    result = {"workload": spec["what"], "B": B, "NB": NB, "kv_tokens": int(T.sum()), "kv_pools_rotated": n_layers,
              "dtype": wl.dtype}
    # ---- timed region (the headline workload only)
    if timed:
        for t in range(args.warmup):
            run_step(t)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for t in range(args.steps):
            run_step(args.warmup + t)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        result["ms_per_step"] = elapsed / args.steps * 1e3
        result["timed_region_s"] = elapsed
        result["query_tokens_per_step"] = int(sum(sum(v) for v in tokens_of.values()))
        assert int(state.fault.item()) == 0

    # ---- dispatch floor: back-to-back launches of a kernel that does nothing to speak of (a one-element
    # fill), timed the same way.  A call whose traffic at 8 TB/s takes less than this (configs 1-2) is bound
    # by it, not by HBM: per_call reports max(bytes / 8 TB/s, floor) next to the plain figure.
    REP = max(20, n_layers)
    tiny = torch.zeros(1, dtype=torch.float32, device=dev)

    def timed_runner(body, reps=5):
        body()
        runner = body
        if not args.no_graph:
            gk = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gk):
                body()
            runner = gk.replay
        runner()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            runner()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e-3 / REP)
        return times

    def floor_body():
        for _ in range(REP):
            tiny.fill_(1.0)

    dispatch_floor = float(np.mean(timed_runner(floor_body, reps=3)))
    result["dispatch_floor_us"] = round(dispatch_floor * 1e6, 2)

    # ---- average launch of each kind of attention call: REP back-to-back launches of the call (state
    # restored to what that call sees, its step's plan as the metadata call left it)
    per_call = {}
    for kind, (st_snap, c) in snaps.items():
        _, stage, new_len, step, q, fn = c

        def body():
            for dst, src in zip(live, st_snap):
                dst.copy_(src)
            for _ in range(REP):
                fn(next_kv(), state, step, q, ws, out=outs[id(c)])

        times = timed_runner(body)
        avg = float(np.mean(times))
        bts = float(np.mean(bytes_of[kind]))
        ntok = float(np.mean(tokens_of[kind]))
        bound = max(bts / (HBM_PEAK_GBS * 1e9), dispatch_floor)
        entry = {"launches_per_step": len(bytes_of[kind]), "avg_us": round(avg * 1e6, 2),
                 "min_us": round(float(np.min(times)) * 1e6, 2), "query_tokens_per_launch": int(ntok),
                 "query_tokens_per_s": round(ntok / avg, 1), "algorithmic_MB": round(bts / 1e6, 3),
                 "GBps": round(bts / avg / 1e9, 1), "frac_of_8TBps": round(bts / avg / 1e9 / HBM_PEAK_GBS, 4),
                 "latency_aware_bound_us": round(bound * 1e6, 2), "frac_of_latency_aware_bound": round(bound / avg, 4)}
        if kind == "chunk":
            entry["TFLOPs"] = round(chunk_flops / avg / 1e12, 1)
            entry["frac_of_bf16_mfma_peak"] = round(chunk_flops / avg / 1e12 / MFMA_BF16_TFLOPS, 4)
            entry["algorithmic_GFLOP"] = round(chunk_flops / 1e9, 1)
        tr = profile_figure(name, kind)
        if tr is not None:
            entry["hbm_traffic_MB_counters"] = round(tr / 1e6, 1)
        per_call[kind] = entry

    if args.extras or (name == HEADLINE and args.workload == "all"):
        extras(name, args, mods, locals(), per_call)
    result["per_call"] = per_call
    result["_wl"] = (wl, base_len, C)
    return result


def profile_figure(workload, kind):
    """HBM bytes per launch as the counters saw them: the figure of the committed rocprofv3 summary of this
    workload (a line "traffic_bytes_per_<kind>_launch = N" in profiles/attn_<workload>_hbm_traffic.md), None
    when there is none."""
    path = os.path.join(ROOT, "profiles", f"attn_{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    m = re.search(rf"^traffic_bytes_per_{kind}_launch\s*=\s*(\d+)", open(path).read(), re.M)
    return int(m.group(1)) if m else None


def extras(name, args, mods, env, per_call):
    """Two more launches around the hot path, outside the timed step: the rotary encoding + cache append of the
    parallel-decode rows, and a mixed step (half of the sequences serial, half in their parallel stage)."""
    np, torch, W, A = mods
    wl, kv, state, snaps, live, ws, dev, B = (env[k] for k in ("wl", "kv", "state", "snaps", "live", "ws", "dev", "B"))
    timed_runner, next_kv, rand_q, dev_i32, REP, bytes_of = (env[k] for k in ("timed_runner", "next_kv", "rand_q", "dev_i32",
                                                                            "REP", "bytes_of"))
    st_snap, c = snaps["parallel"]
    step_p, q_p = c[3], c[4].clone()
    k_new = (torch.randn(step_p.NQ, wl.num_kv_heads, wl.head_dim, device=dev) * wl.sigma).to(wl.torch_dtype)
    v_new = (torch.randn(step_p.NQ, wl.num_kv_heads, wl.head_dim, device=dev) * wl.sigma).to(wl.torch_dtype)

    def rope_body():
        for _ in range(REP):
            A.aspd_rope_append(kv, step_p, q_p, k_new, v_new, 1e6)

    per_call["rope_append"] = {"launches_per_step": 0, "avg_us": round(float(np.mean(timed_runner(rope_body, reps=2))) * 1e6, 2),
                               "query_tokens_per_launch": int(step_p.NQ),
                               "note": "rows of the parallel-decode call; outside the timed step"}
    if B < 2:
        return
    for dst, src in zip(live, st_snap):
        dst.copy_(src)
    ending = np.array([1 if s < B // 2 else 0 for s in range(B)], dtype=np.int32)
    A.aspd_build_branch_meta(kv, state, A.STAGE_MERGE, dev_i32(ending))
    keep = np.where(ending == 1, 0, wl.num_branches).astype(np.int64)
    new_cu = np.zeros(B + 1, dtype=np.int32)
    np.cumsum(keep, out=new_cu[1:])
    A.aspd_renumber_branches(state, torch.from_numpy(new_cu))
    nb2 = int(new_cu[-1])
    mixed_len = dev_i32(np.concatenate([np.ones(nb2), ending]))
    nq_mixed = nb2 + int(ending.sum())
    step_m = A.aspd_build_branch_meta(kv, state, A.STAGE_MIXED, mixed_len, NQ=nq_mixed, max_new_per_seq=int(max(keep.max(), 1)))
    q_m = rand_q(nq_mixed)
    out_m = torch.empty_like(q_m)

    def mixed_body():
        for _ in range(REP):
            A.aspd_attn_parallel_decode(next_kv(), state, step_m, q_m, ws, out=out_m)

    avg = float(np.mean(timed_runner(mixed_body, reps=2)))
    bts = float(bytes_of["parallel"][0])
    per_call["mixed"] = {"launches_per_step": 0, "avg_us": round(avg * 1e6, 2), "query_tokens_per_launch": nq_mixed,
                         "algorithmic_MB": round(bts / 1e6, 3), "GBps": round(bts / avg / 1e9, 1),
                         "note": f"{int(ending.sum())} sequences serial, {B - int(ending.sum())} in their parallel stage, "
                                 "one launch; outside the timed step"}
    assert int(state.fault.item()) == 0
    if wl.dtype != "bf16":
        return
    # whole sequences (teacher forcing, re-prefill): every token of the batch a query row, one launch
    layouts = W.random_layouts(wl, seed=17, max_branches=10, fill=0.97)
    cu = np.zeros(B + 1, dtype=np.int32)
    np.cumsum([len(r) for r in layouts], out=cu[1:])
    br = np.array([b for r in layouts for b, _ in r], dtype=np.int32)
    ln = np.array([n for r in layouts for _, n in r], dtype=np.int32)
    nq_all = int(ln.sum())
    st2 = A.BatchState(B, state.owner_stride, dev)
    step_s = A.aspd_build_sequence_meta(kv, st2, dev_i32(cu), dev_i32(br), dev_i32(ln), NQ=nq_all)
    q_s = rand_q(nq_all)
    out_s = torch.empty_like(q_s)
    keys = int(step_s.kv_len[:nq_all].to(torch.int64).sum().item())
    flops = keys * 4 * wl.head_dim * wl.num_q_heads

    def seq_body():
        for _ in range(REP):
            A.aspd_attn_full_sequence(next_kv(), st2, step_s, q_s, ws, out=out_s)

    avg = float(np.mean(timed_runner(seq_body, reps=2)))
    assert int(st2.fault.item()) == 0
    per_call["full_sequence"] = {"launches_per_step": 0, "avg_us": round(avg * 1e6, 1), "query_tokens_per_launch": nq_all,
                                 "query_tokens_per_s": round(nq_all / avg, 1), "algorithmic_GFLOP": round(flops / 1e9, 1),
                                 "TFLOPs": round(flops / avg / 1e12, 1),
                                 "frac_of_bf16_mfma_peak": round(flops / avg / 1e12 / MFMA_BF16_TFLOPS, 4),
                                 "note": "all tokens of the batch as query rows under the mask of Eq. 2-3 (serial and "
                                         "parallel stages alternating, branches laid one after the other); flops count "
                                         "visible keys only; outside the timed step"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="all", choices=["all"] + sorted(WORKLOADS),
                    help="all: the five configurations, headline configuration 5; one name: that workload alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="distinct KV pools to rotate through (0 = enough for 1.5 GB)")
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying a HIP graph")
    ap.add_argument("--extras", action="store_true", help="also time the rotary append, a mixed step and the whole-sequence call (the default run does so for the headline workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is one-GPU only (the path shards by sequence or KV head without "
              "exchange, nothing here uses a second GPU); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import aspd_workloads as W
    from paper_2508_08895_amd import binding as A

    A.lib()  # fail loudly when the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    mods = (np, torch, W, A)
    dev = torch.device("cuda:0")

    names = DEFAULT_SET if args.workload == "all" else (args.workload,)
    head_name = HEADLINE if args.workload == "all" else args.workload
    results = {}
    for name in names:
        results[name] = measure(name, args, timed=(name == head_name), mods=mods)
        if name != head_name:
            results[name].pop("_wl")
        torch.cuda.empty_cache()
    head = results[head_name]
    wl, base_len, C = head.pop("_wl")

    # ---- what a plain read-only stream reaches on this device (2 GiB, larger than any cache)
    probe_src = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    probe_src.zero_()
    probe_sink = torch.empty(64 << 10, dtype=torch.uint8, device=dev)
    for _ in range(2):
        A.aspd_probe_read_bandwidth(probe_src, probe_sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        A.aspd_probe_read_bandwidth(probe_src, probe_sink)
    e1.record()
    torch.cuda.synchronize()
    read_ceiling = 5 * probe_src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del probe_src

    # ---- the dominant kernel of the metric: the parallel-decode launch of the headline workload, alone
    par = head["per_call"]["parallel"]
    roofline = {"bound": "hbm", "kernel": f"attn_bf16_kernel, parallel-decode launch of {head_name}",
                "achieved": par["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": par["frac_of_8TBps"],
                "traffic": profile_figure(head_name, "parallel"),
                "traffic_source": f"profiles/attn_{head_name}_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command)",
                "avg_launch_us": par["avg_us"], "algorithmic_bytes_per_launch": int(par["algorithmic_MB"] * 1e6),
                "plain_read_stream_GBps": round(read_ceiling, 1),
                "frac_of_plain_read_stream": round(par["GBps"] / read_ceiling, 4),
                "dispatch_floor_us": head["dispatch_floor_us"]}
    roofline_chunk = None
    if "chunk" in head["per_call"]:
        ch = head["per_call"]["chunk"]
        roofline_chunk = {"bound": "mfma", "kernel": f"attn_bf16_rows_kernel, branch-chunk launch of {head_name}",
                          "achieved": ch["TFLOPs"], "peak": MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                          "frac": ch["frac_of_bf16_mfma_peak"], "avg_launch_us": ch["avg_us"],
                          "algorithmic_GFLOP": ch["algorithmic_GFLOP"],
                          "hbm": {"algorithmic_MB": ch["algorithmic_MB"], "GBps": ch["GBps"], "frac_of_8TBps": ch["frac_of_8TBps"],
                                  "traffic": profile_figure(head_name, "chunk")}}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, base_len, C, np)

    per_config = {}
    for name, r in results.items():
        per_config[name] = {k: v for k, v in r.items() if k not in ("ms_per_step", "timed_region_s", "query_tokens_per_step")}
    line = {"metric": "branch-query tokens/s of the parallel-decode attention call, one attention layer "
                      "(achieved HBM GB/s and fraction of 8 TB/s in roofline and per_config)",
            "value": par["query_tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(head["ms_per_step"], 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
            "data": "synthetic", "launch": "eager" if args.no_graph else "hip_graph",
            "config": {"workload": f"{head_name}: {WORKLOADS[head_name]['what']}",
                       "value_is": "branch queries of one parallel-decode launch / its average duration (per_config."
                                   f"{head_name}.per_call.parallel)",
                       "step_is": "the whole hot path on this batch: " + WORKLOADS[head_name]["what"].split(": ", 1)[-1],
                       "query_tokens_per_step": head["query_tokens_per_step"], "B": head["B"], "NB": head["NB"],
                       "kv_tokens": head["kv_tokens"], "kv_pools_rotated": head["kv_pools_rotated"],
                       "timed_region_s": round(head["timed_region_s"], 3)},
            "per_config": per_config, "roofline": roofline, "roofline_chunk": roofline_chunk, "cpu_baseline": cpu}
    print(json.dumps(line), flush=True)
    return 0


def cpu_baseline(wl, base_len, chunk, np):
    """The oracle as it stands, timed on this host for the parallel-decode call of the workload."""
    from oracle import TokenTable
    from oracle import attention_c
    tt = TokenTable(wl.block_tables, wl.block_size)
    tt.append_serial(wl.prefix_len)
    tt.open_parallel(wl.num_branches)
    target = base_len + chunk
    max_steps = int(min(8, target.min()))   # the timed steps end where the GPU's parallel-decode call stands
    # replay cheaply: one multi-token append per branch gives the same token set per branch; the
    # arrangement differs from the interleaved one but the oracle's cost and result shape do not
    tt.append_parallel(target + 1 - max(max_steps, 1))
    ones = np.ones(wl.NB, dtype=np.int32)
    # consecutive parallel-decode steps (metadata + attention each) until about ten seconds have passed
    t0 = time.perf_counter()
    done = total = steps = 0
    while steps < max(max_steps, 1) and time.perf_counter() - t0 < 15.0:
        meta = tt.append_parallel(ones)
        q = wl.draw_q(meta.NQ)
        rows = None
        if meta.NQ > 192:  # bound the work: a seeded sample of the rows
            rows = np.sort(np.random.default_rng(1 + steps).choice(meta.NQ, size=192, replace=False))
        attention_c.attend_c(tt, meta, q, wl.k_cache, wl.v_cache, rows=rows)
        done += meta.NQ if rows is None else len(rows)
        total += meta.NQ
        steps += 1
    dt = time.perf_counter() - t0
    return {"value": round(done / dt, 3), "unit": "tokens/s", "cores": int(attention_c.last_threads), "kind": "oracle",
            "implementation": "oracle/attention_ref.c: plain C loops, float64, explicit dense mask, OpenMP over (row, head), "
                              "no BLAS; metadata and mask from the Python token table",
            "sample": f"{steps} consecutive parallel-decode calls: {done} of {total} branch queries x "
                      f"{wl.num_q_heads} heads, metadata + float64 dense-mask attention, {dt:.1f}s"}


if __name__ == "__main__":
    sys.exit(main())
