// aspd_build_branch_meta: position ids (ASPD Sec. 3.2, Eq. 4), cache slots and owner tags for the
// tokens one append call adds, and the update of the batch's decode state (Sec. 3.3 stage switches).
//
// Pure integer work, one workgroup per sequence.  A workgroup needs two things from outside its own
// sequence: the packed row of its first token (the number of tokens appended to earlier sequences)
// and nothing else, so it sums new_len over the earlier branches itself instead of waiting for a
// batch-wide scan: new_len is an input no workgroup writes, hence no ordering between workgroups.
#include "aspd_plan.h"

namespace {

constexpr int META_THREADS = 256;

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Sum over the workgroup; every thread gets the total.  `red` holds META_THREADS/64 ints.
__device__ int block_sum(int v, int* red) {
  v = wave_sum(v);
  __syncthreads();  // red may still be read from an earlier call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  int tot = 0;
#pragma unroll
  for (int w = 0; w < META_THREADS / 64; ++w) tot += red[w];
  return tot;
}

__device__ __forceinline__ void raise_fault(int32_t* fault, int bits) {
  if (fault) atomicOr(fault, bits);
}

// PARALLEL stage: new_len[NB].  Branch tokens take position stage_start + index-in-branch (Eq. 4,
// second case) and are laid at the tail of the sequence ordered by (branch, token).
// MIXED: main_len[B] as well.  Sequences switch between serial and parallel decoding independently
// (Sec. 3.3), so one call may serve sequences with open branches (their branch entries of new_len)
// and sequences without (their entry of main_len: main-branch tokens, Eq. 4 first case).
// Position paradigms (Sec. 4.5.3): under Same-Seq the main branch's position counter is the token count
// and needs no storage; under Same-Max and fixed intervals it lives in st.main_pos.  `fix_n` > 0
// selects fixed intervals of that many positions per branch.
__global__ __launch_bounds__(META_THREADS) void meta_parallel_kernel(KvView kv, StateView st, StepView sp,
                                                                     const int32_t* __restrict__ new_len,
                                                                     const int32_t* __restrict__ main_len,
                                                                     bool same_seq, int fix_n) {
  __shared__ int red[META_THREADS / 64];
  __shared__ int off[ASPD_MAX_BRANCHES_PER_SEQ + 2];  // exclusive scan of this sequence's new_len
  __shared__ int held[ASPD_MAX_BRANCHES_PER_SEQ + 1]; // tokens each branch already holds
  const int s = blockIdx.x;
  const int tid = threadIdx.x;
  const int b0 = st.cu_branches[s];
  const int b1 = st.cu_branches[s + 1];
  const int L = st.stage_base[s];  // state is read here, ahead of the barriers below, and
  const int T = st.seq_len[s];     // written only after the last of them
  // position the next main-branch token takes = position of the first token of every branch of a
  // stage that opens now (stage_start of Eq. 4); it does not move while the stage runs
  const int P = same_seq ? L : st.main_pos[s];
  int K = b1 - b0;
  if (K > ASPD_MAX_BRANCHES_PER_SEQ) {
    if (tid == 0) raise_fault(st.fault, ASPD_FAULT_BRANCHES);
    K = ASPD_MAX_BRANCHES_PER_SEQ;
  }

  // packed row of this sequence's first new token
  int part = 0;
  for (int i = tid; i < b0; i += META_THREADS) part += new_len[i];
  if (main_len)
    for (int i = tid; i < s; i += META_THREADS) part += main_len[i];
  const int base = block_sum(part, red);
  const int c_main = main_len ? main_len[s] : 0;

  if (K == 0) {
    // no open branch: the sequence is serial and takes main-branch tokens (or none)
    if (tid == 0) {
      sp.cu_seq_new[s] = base;
      if (s == st.B - 1) {
        sp.cu_seq_new[st.B] = base + c_main;
        sp.cu_new[b1] = base + c_main;
      }
    }
    bool ok = true;
    if ((long)T + c_main > (long)kv.max_blocks_per_seq * ASPD_BLOCK) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE); }
    if (base + c_main > sp.NQ) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_ROW_COUNT); }
    if (c_main > 0 && (L != T || (st.stage_open && st.stage_open[s]))) {  // unmerged stage
      ok = false;
      if (tid == 0) raise_fault(st.fault, ASPD_FAULT_STAGE);
    }
    if (!ok || c_main == 0) return;
    for (int idx = tid; idx < c_main; idx += META_THREADS) {
      const int row = base + idx;
      const int slot = T + idx;
      const int blk = kv.block_tables[(long)s * kv.max_blocks_per_seq + slot / ASPD_BLOCK];
      if (blk < 0 || blk >= kv.num_blocks) raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE);
      sp.q_seq[row] = s;
      sp.q_branch[row] = -1;
      sp.position_ids[row] = (same_seq ? T : P) + idx;
      sp.logical_slot[row] = slot;
      sp.slot_mapping[row] = (int64_t)blk * ASPD_BLOCK + slot % ASPD_BLOCK;
      sp.kv_len[row] = slot + 1;
    }
    if (tid == 0) {  // T and L were read before any barrier; nobody else touches this sequence
      st.seq_len[s] = T + c_main;
      st.stage_base[s] = T + c_main;
      if (st.main_pos) st.main_pos[s] = (same_seq ? T : P) + c_main;
    }
    return;
  }
  if (c_main != 0) {  // main-branch tokens while branches are open: refuse the sequence
    if (tid == 0) raise_fault(st.fault, ASPD_FAULT_STAGE);
    return;
  }
  if (tid == 0 && st.stage_open) st.stage_open[s] = 1;  // named with branches: in a parallel stage, tokens or not

  // scan over the sequence's own branches (K <= 255: one branch per thread, serial scan by thread 0
  // would do, but a log-step scan keeps the launch short for wide stages)
  const int c_mine = (tid < K) ? new_len[b0 + tid] : 0;
  if (tid < K) held[tid] = st.branch_len[b0 + tid];
  if (tid <= K) off[tid] = 0;
  __syncthreads();
  {
    // inclusive Hillis-Steele in registers + LDS over the first 256 threads
    __shared__ int scan[META_THREADS];
    scan[tid] = c_mine;
    __syncthreads();
    for (int d = 1; d < META_THREADS; d <<= 1) {
      int v = (tid >= d) ? scan[tid - d] : 0;
      __syncthreads();
      scan[tid] += v;
      __syncthreads();
    }
    if (tid < K) off[tid + 1] = scan[tid];
    __syncthreads();
  }
  const int total = off[K];

  if (tid < K) sp.cu_new[b0 + tid] = base + off[tid];
  if (tid == 0) {
    sp.cu_seq_new[s] = base;
    if (s == st.B - 1) {
      sp.cu_seq_new[st.B] = base + total;
      sp.cu_new[b1] = base + total;
    }
  }

  // capacity of this sequence in slots
  const long cap_slots = (long)kv.max_blocks_per_seq * ASPD_BLOCK;
  bool ok = true;
  if ((long)T + total > cap_slots) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE); }
  if ((long)T + total > st.owner_stride) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_OWNER_ROW); }
  if (base + total > sp.NQ) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_ROW_COUNT); }
  if (fix_n > 0 && __syncthreads_or(tid < K && held[tid] + c_mine > fix_n)) {
    ok = false;
    if (tid == 0) raise_fault(st.fault, ASPD_FAULT_INTERVAL);
  }
  if (!ok) return;  // the sequence is left as it was

  for (int idx = tid; idx < total; idx += META_THREADS) {
    // branch of token idx: last k with off[k] <= idx
    int lo = 0, hi = K - 1;
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (off[mid] <= idx) lo = mid; else hi = mid - 1;
    }
    const int k = lo;
    const int t = held[k] + (idx - off[k]);  // 0-based index of the token within its branch
    const int row = base + idx;
    const int slot = T + idx;
    const int blk = kv.block_tables[(long)s * kv.max_blocks_per_seq + slot / ASPD_BLOCK];
    if (blk < 0 || blk >= kv.num_blocks) raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE);
    sp.q_seq[row] = s;
    sp.q_branch[row] = b0 + k;
    sp.position_ids[row] = P + k * fix_n + t;
    sp.logical_slot[row] = slot;
    sp.slot_mapping[row] = (int64_t)blk * ASPD_BLOCK + slot % ASPD_BLOCK;
    sp.kv_len[row] = L + t + 1;  // shared prefix + own branch up to and including itself
    st.slot_owner[(long)s * st.owner_stride + slot] = (uint8_t)(k + 1);
  }
  // state update: every read of branch_len / seq_len happened before the barriers of the scan
  __syncthreads();
  if (tid < K) st.branch_len[b0 + tid] = held[tid] + c_mine;
  if (tid == 0) st.seq_len[s] = T + total;
}

// SERIAL stage: new_len[B].  A main-branch token's position is the number of tokens decoded before
// it, all branches of all earlier stages included (Eq. 4, first case): its flattened index.
__global__ __launch_bounds__(META_THREADS) void meta_serial_kernel(KvView kv, StateView st, StepView sp,
                                                                   const int32_t* __restrict__ new_len, bool same_seq) {
  __shared__ int red[META_THREADS / 64];
  const int s = blockIdx.x;
  const int tid = threadIdx.x;
  int part = 0;
  for (int i = tid; i < s; i += META_THREADS) part += new_len[i];
  const int base = block_sum(part, red);
  const int c = new_len[s];
  const int T = st.seq_len[s];
  const int L = st.stage_base[s];
  const int P = same_seq ? T : st.main_pos[s];
  const bool open = st.stage_open && st.stage_open[s];
  if (tid == 0) {
    sp.cu_new[s] = base;
    sp.cu_seq_new[s] = base;
    if (s == st.B - 1) {
      sp.cu_new[st.B] = base + c;
      sp.cu_seq_new[st.B] = base + c;
    }
  }
  bool ok = true;
  if ((long)T + c > (long)kv.max_blocks_per_seq * ASPD_BLOCK) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE); }
  if (base + c > sp.NQ) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_ROW_COUNT); }
  // A main-branch token under a parallel stage that has not been merged would take a position inside the
  // branches' range (Eq. 4 case 1 counts the tokens of finished stages only): refuse the sequence.
  if (c > 0 && (L != T || open)) { ok = false; if (tid == 0) raise_fault(st.fault, ASPD_FAULT_STAGE); }
  if (!ok) return;
  for (int idx = tid; idx < c; idx += META_THREADS) {
    const int row = base + idx;
    const int slot = T + idx;
    const int blk = kv.block_tables[(long)s * kv.max_blocks_per_seq + slot / ASPD_BLOCK];
    if (blk < 0 || blk >= kv.num_blocks) raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE);
    sp.q_seq[row] = s;
    sp.q_branch[row] = -1;
    sp.position_ids[row] = P + idx;
    sp.logical_slot[row] = slot;
    sp.slot_mapping[row] = (int64_t)blk * ASPD_BLOCK + slot % ASPD_BLOCK;
    sp.kv_len[row] = slot + 1;
  }
  __syncthreads();
  if (tid == 0) {
    st.seq_len[s] = T + c;
    st.stage_base[s] = T + c;  // a serial sequence has no branch region
    if (st.main_pos) st.main_pos[s] = P + c;
  }
}

// MERGE: the parallel stage ends.  Everything decoded so far becomes visible to all later queries;
// the cache is reused as it is (Sec. 3.3: no re-prefill when switching back).
__global__ void meta_merge_kernel(StateView st, const int32_t* __restrict__ which /* null: every sequence */,
                                  bool same_seq, int fix_n) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= st.B || (which && which[s] == 0)) return;
  const int T = st.seq_len[s];
  const bool running = st.stage_base[s] < T;
  const bool open = st.stage_open ? st.stage_open[s] != 0 : running;
  st.stage_base[s] = T;
  if (st.stage_open) st.stage_open[s] = 0;
  if (!st.main_pos) return;
  // where the main branch continues (Sec. 4.5.3)
  if (same_seq) {
    st.main_pos[s] = T;
  } else if (st.cu_branches) {
    const int b0 = st.cu_branches[s], K = st.cu_branches[s + 1] - b0;
    if (fix_n > 0) {
      // the K intervals were allotted when the stage opened and are spent, tokens or not
      if (open) st.main_pos[s] += K * fix_n;
    } else if (running) {
      int longest = 0;
      for (int k = 0; k < K; ++k) longest = max(longest, st.branch_len[b0 + k]);
      st.main_pos[s] += longest;  // right after the largest position a branch reached
    }
  }
}

// Branch numbering changes when sequences open or end stages at different times: the tokens held by
// the branches of stages still running move to their branches' new indices, every other entry starts
// at zero.  A stage is running while stage_base < seq_len (one that holds no token yet has only zeros).
// Every sequence that is given branches is in a parallel stage from here on (stage_open).
__global__ void meta_renumber_kernel(StateView st, const int32_t* __restrict__ new_cu,
                                     int32_t* __restrict__ new_len_held) {
  const int s = blockIdx.x;
  const int o0 = st.cu_branches[s], k_old = st.cu_branches[s + 1] - o0;
  const int n0 = new_cu[s], k_new = new_cu[s + 1] - n0;
  const bool running = st.stage_base[s] < st.seq_len[s];
  if (running && k_new != k_old) {
    if (threadIdx.x == 0) raise_fault(st.fault, ASPD_FAULT_STAGE);
    return;
  }
  for (int k = threadIdx.x; k < k_new; k += blockDim.x) new_len_held[n0 + k] = running ? st.branch_len[o0 + k] : 0;
  if (threadIdx.x == 0 && st.stage_open) st.stage_open[s] = k_new > 0 ? 1 : 0;
}

}  // namespace

int aspd_check_kv(const aspd_kv* kv) {
  if (!kv || !kv->k_cache_d || !kv->v_cache_d || !kv->block_tables_d) return ASPD_ERR_INVALID_ARG;
  if (kv->num_blocks <= 0 || kv->max_blocks_per_seq <= 0 || kv->num_q_heads <= 0 || kv->num_kv_heads <= 0)
    return ASPD_ERR_INVALID_ARG;
  if (kv->block_size != ASPD_BLOCK) return ASPD_ERR_UNSUPPORTED;
  if (kv->head_dim != 64 && kv->head_dim != 128) return ASPD_ERR_UNSUPPORTED;
  if (kv->dtype != ASPD_F32 && kv->dtype != ASPD_BF16) return ASPD_ERR_UNSUPPORTED;
  if (kv->num_q_heads % kv->num_kv_heads != 0) return ASPD_ERR_UNSUPPORTED;
  if (((uintptr_t)kv->k_cache_d & 15) || ((uintptr_t)kv->v_cache_d & 15)) return ASPD_ERR_INVALID_ARG;
  return ASPD_OK;
}

extern "C" int aspd_build_branch_meta(const aspd_kv* kv, aspd_state* state, int32_t stage, int32_t pos_mode,
                                      const int32_t* new_len_d, aspd_step* out, void* stream) {
  int rc = aspd_check_kv(kv);
  if (rc != ASPD_OK) return rc;
  if (!state || state->B <= 0 || !state->stage_base_d || !state->seq_len_d) return ASPD_ERR_INVALID_ARG;
  if (state->B > ASPD_MAX_BATCH) return ASPD_ERR_UNSUPPORTED;
  const bool same_seq = pos_mode == ASPD_POS_SAME_SEQ;
  const int fix_n = (pos_mode & 0xff) == 2 ? (pos_mode >> 8) : 0;
  if (!same_seq && pos_mode != ASPD_POS_SAME_MAX && fix_n <= 0) return ASPD_ERR_UNSUPPORTED;
  if (!same_seq && !state->main_pos_d) return ASPD_ERR_INVALID_ARG;
  if (fix_n > 0 && !state->stage_open_d) return ASPD_ERR_INVALID_ARG;
  hipStream_t hs = (hipStream_t)stream;
  StateView sv = make_view(state);

  if (stage == ASPD_STAGE_MERGE) {
    hipLaunchKernelGGL(meta_merge_kernel, dim3((state->B + 255) / 256), dim3(256), 0, hs, sv, new_len_d, same_seq,
                       fix_n);
    ASPD_HIP_CHECK(hipGetLastError());
    return ASPD_OK;
  }
  if (stage != ASPD_STAGE_PARALLEL && stage != ASPD_STAGE_SERIAL && stage != ASPD_STAGE_MIXED)
    return ASPD_ERR_INVALID_ARG;
  if (!new_len_d || !out || out->NQ < 0) return ASPD_ERR_INVALID_ARG;
  if (!out->cu_new_d || !out->cu_seq_new_d) return ASPD_ERR_INVALID_ARG;
  if (out->NQ > 0 && (!out->q_seq_d || !out->q_branch_d || !out->position_ids_d || !out->logical_slot_d ||
                      !out->slot_mapping_d || !out->kv_len_d))
    return ASPD_ERR_INVALID_ARG;
  if (out->max_new_per_seq < 0 || out->max_workgroups < 0) return ASPD_ERR_INVALID_ARG;
  // the plan of the step's attention launches, for the launch shape the step's hints select
  AttnVariant variant;
  bool with_plan = false;
  out->plan_key = 0;
  if (out->plan_d && out->NQ > 0 &&
      aspd_choose_variant(kv, state->B, out->NQ, out->max_new_per_seq, out->max_workgroups, false,
                          stage != ASPD_STAGE_SERIAL && out->shared_mask == 0, &variant)) {
    if (((uintptr_t)out->plan_d & 255) ||
        out->plan_bytes < aspd_plan_words(kv, variant, state->B, out->NQ) * sizeof(int32_t))
      return ASPD_ERR_INVALID_ARG;
    with_plan = true;
  }
  KvView kvv = make_view(kv);
  StepView spv = make_view(out);
  if (stage == ASPD_STAGE_PARALLEL || stage == ASPD_STAGE_MIXED) {
    if (state->NB < (stage == ASPD_STAGE_PARALLEL ? 1 : 0) || !state->cu_branches_d || !state->branch_len_d ||
        !state->slot_owner_d || state->owner_stride <= 0)
      return ASPD_ERR_INVALID_ARG;
    const int32_t* main_len_d = stage == ASPD_STAGE_MIXED ? new_len_d + state->NB : nullptr;
    hipLaunchKernelGGL(meta_parallel_kernel, dim3(state->B), dim3(META_THREADS), 0, hs, kvv, sv, spv, new_len_d,
                       main_len_d, same_seq, fix_n);
  } else {
    hipLaunchKernelGGL(meta_serial_kernel, dim3(state->B), dim3(META_THREADS), 0, hs, kvv, sv, spv, new_len_d,
                       same_seq);
  }
  ASPD_HIP_CHECK(hipGetLastError());
  if (with_plan) {
    rc = aspd_plan_launch(kv, variant, state->B, state->stage_base_d, state->seq_len_d, out->cu_seq_new_d,
                          out->plan_d, hs);
    if (rc != ASPD_OK) return rc;
    out->plan_key = aspd_plan_key(variant, state->B);
  }
  return ASPD_OK;
}

extern "C" int aspd_renumber_branches(const aspd_state* state, const int32_t* new_cu_branches_d,
                                      int32_t* new_branch_len_d, void* stream) {
  if (!state || state->B <= 0 || !state->stage_base_d || !state->seq_len_d || !state->cu_branches_d ||
      !state->branch_len_d || !new_cu_branches_d || !new_branch_len_d)
    return ASPD_ERR_INVALID_ARG;
  if (state->B > ASPD_MAX_BATCH) return ASPD_ERR_UNSUPPORTED;
  if (new_cu_branches_d == state->cu_branches_d || new_branch_len_d == state->branch_len_d)
    return ASPD_ERR_INVALID_ARG;  // the old arrays are read while the new ones are written
  hipLaunchKernelGGL(meta_renumber_kernel, dim3(state->B), dim3(64), 0, (hipStream_t)stream, make_view(state),
                     new_cu_branches_d, new_branch_len_d);
  ASPD_HIP_CHECK(hipGetLastError());
  return ASPD_OK;
}

extern "C" const char* aspd_status_string(int status) {
  switch (status) {
    case ASPD_OK: return "ok";
    case ASPD_ERR_INVALID_ARG: return "invalid argument";
    case ASPD_ERR_UNSUPPORTED: return "unsupported configuration";
    case ASPD_ERR_WORKSPACE: return "workspace too small";
    case ASPD_ERR_HIP: return "HIP call failed";
    case ASPD_ERR_SCRATCH_LIMIT: return "call needs more scratch than the library's static array holds";
    default: return "unknown status";
  }
}
