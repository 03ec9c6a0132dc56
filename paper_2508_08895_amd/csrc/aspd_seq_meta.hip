// aspd_build_sequence_meta: metadata of ALL tokens of a batch of multi-stage sequences at once
// (ASPD Fig. 5, training arrangement: the branches of a parallel stage laid one after the other;
// Eq. 4 for the position ids, Eq. 2-3 for what a token sees), for teacher-forced passes and for the
// re-prefill of a cache (Sec. 4.5.3, "Same-Re").
//
// Pure integer work.  One workgroup per sequence: one thread walks the sequence's runs in order (a
// few hundred at most: the walk carries the stage bookkeeping, which is inherently sequential) and
// tabulates, per run, its first slot, the position of its first token, the first slot of its stage
// and its branch number; then all threads emit the tokens, finding a token's run by binary search.
// A second, one-workgroup kernel lists the row groups of the attention launch, longest key range
// first, behind the per-row stage bases in the step's plan buffer.
#include "aspd_plan.h"

namespace {

constexpr int SEQ_META_THREADS = 256;

__device__ __forceinline__ void seq_raise_fault(int32_t* fault, int bits) {
  if (fault) atomicOr(fault, bits);
}

struct LayoutView {
  const int32_t* cu_runs;
  const int32_t* run_branch;
  const int32_t* run_len;
};

__global__ __launch_bounds__(SEQ_META_THREADS) void meta_sequence_kernel(KvView kv, StateView st, StepView sp,
                                                                         LayoutView lay, int32_t* __restrict__ plan,
                                                                         bool same_seq, bool same_max, int fix_n) {
  __shared__ int run_slot0[ASPD_MAX_RUNS_PER_SEQ + 1];  // first slot of every run; [nr] = tokens of the sequence
  __shared__ int run_pos0[ASPD_MAX_RUNS_PER_SEQ];       // position id of the run's first token
  __shared__ int run_base[ASPD_MAX_RUNS_PER_SEQ];       // first slot of the run's stage (branch runs)
  __shared__ int red[SEQ_META_THREADS / 64];
  __shared__ int sh_ok;
  const int s = blockIdx.x;
  const int tid = threadIdx.x;
  const int r0 = lay.cu_runs[s];
  const int nr = lay.cu_runs[s + 1] - r0;

  // packed row of this sequence's first token: the tokens of all earlier sequences
  int part = 0;
  for (int i = tid; i < r0; i += SEQ_META_THREADS) part += max(lay.run_len[i], 0);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
  if ((tid & 63) == 0) red[tid >> 6] = part;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < SEQ_META_THREADS / 64; ++w) base += red[w];

  if (tid == 0) {
    int ok = 1, faults = 0;
    int slot = 0;         // tokens laid so far
    int main_pos = 0;     // position the next main-branch token takes (Same-Seq: equals `slot` outside stages)
    int stage_first = 0;  // first slot of the running parallel stage
    int stage_start = 0;  // Eq. 4 stage_start: position of the first token of each of its branches
    int longest = 0;      // most tokens any of its branches holds
    int prev = 0;         // branch number of the previous run (0: main branch)
    if (nr < 0 || nr > ASPD_MAX_RUNS_PER_SEQ) {
      ok = 0;
      faults |= ASPD_FAULT_LAYOUT;
    }
    for (int i = 0; ok && i < nr; ++i) {
      const int b = lay.run_branch[r0 + i];
      const int n = lay.run_len[r0 + i];
      if (n < 0 || b < 0 || b > ASPD_MAX_BRANCHES_PER_SEQ || (b > 1 && b != prev + 1)) {
        ok = 0;
        faults |= (b > ASPD_MAX_BRANCHES_PER_SEQ) ? ASPD_FAULT_BRANCHES : ASPD_FAULT_LAYOUT;
        break;
      }
      if (prev > 0 && b <= 1) {
        // the stage that `prev` closed ends here: where the main branch continues (Sec. 4.5.3)
        main_pos = same_seq ? slot : (same_max ? stage_start + longest : stage_start + prev * fix_n);
      }
      run_slot0[i] = slot;
      if (b == 0) {
        run_pos0[i] = same_seq ? slot : main_pos;  // Eq. 4, first case
        run_base[i] = slot;
        main_pos = run_pos0[i] + n;
      } else {
        if (b == 1) {  // a stage opens
          stage_first = slot;
          stage_start = same_seq ? slot : main_pos;
          longest = 0;
        }
        if (fix_n > 0 && n > fix_n) {
          ok = 0;
          faults |= ASPD_FAULT_INTERVAL;
          break;
        }
        run_pos0[i] = stage_start + (fix_n > 0 ? (b - 1) * fix_n : 0);  // Eq. 4, second case
        run_base[i] = stage_first;
        longest = max(longest, n);
      }
      slot += n;
      prev = b;
      if ((long)slot > (long)kv.max_blocks_per_seq * ASPD_BLOCK) {
        ok = 0;
        faults |= ASPD_FAULT_BLOCK_TABLE;
      } else if (st.slot_owner && slot > st.owner_stride) {
        ok = 0;
        faults |= ASPD_FAULT_OWNER_ROW;
      }
    }
    if (ok && prev > 0) main_pos = same_seq ? slot : (same_max ? stage_start + longest : stage_start + prev * fix_n);
    if (ok && base + slot > sp.NQ) {
      ok = 0;
      faults |= ASPD_FAULT_ROW_COUNT;
    }
    if (!ok) {
      slot = 0;
      main_pos = 0;
      faults |= ASPD_FAULT_ROW_COUNT;  // the sequence's rows are missing from the step
    }
    if (ok) run_slot0[nr] = slot;
    if (faults) seq_raise_fault(st.fault, faults);
    sh_ok = ok;
    // state: as after a merge of the last stage
    st.seq_len[s] = slot;
    st.stage_base[s] = slot;
    if (st.main_pos) st.main_pos[s] = main_pos;
    if (st.stage_open) st.stage_open[s] = 0;
    sp.cu_seq_new[s] = base;
    if (s == st.B - 1) sp.cu_seq_new[st.B] = base + slot;
  }
  __syncthreads();
  if (!sh_ok) return;
  const int T = run_slot0[nr];
  int32_t* row_base = plan + SEQ_PLAN_HDR;
  for (int j = tid; j < T; j += SEQ_META_THREADS) {
    // the run that holds slot j: the last one whose first slot is <= j and that is not empty
    int lo = 0, hi = nr - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (run_slot0[mid] <= j) lo = mid; else hi = mid - 1;
    }
    const int b = lay.run_branch[r0 + lo];
    const int t = j - run_slot0[lo];  // index of the token within its run (= within its branch)
    const int row = base + j;
    const int blk = kv.block_tables[(long)s * kv.max_blocks_per_seq + j / ASPD_BLOCK];
    if (blk < 0 || blk >= kv.num_blocks) seq_raise_fault(st.fault, ASPD_FAULT_BLOCK_TABLE);
    sp.q_seq[row] = s;
    sp.q_branch[row] = b - 1;
    sp.position_ids[row] = run_pos0[lo] + t;
    sp.logical_slot[row] = j;
    sp.slot_mapping[row] = (int64_t)blk * ASPD_BLOCK + j % ASPD_BLOCK;
    // Eq. 2-3: a main-branch token sees every slot up to its own; a branch token sees everything before
    // its stage and its own branch up to itself
    sp.kv_len[row] = b == 0 ? j + 1 : run_base[lo] + t + 1;
    row_base[row] = b == 0 ? j : run_base[lo];
    if (st.slot_owner) st.slot_owner[(long)s * st.owner_stride + j] = (uint8_t)b;
  }
}

// The row groups of the attention launch: `qpg` consecutive tokens of one sequence each.  A group's key
// range ends at its last token's slot, so groups late in a sequence cost more than early ones; workgroups
// take groups from the list as they become free, and the list starts with the longest ranges so that
// the launch does not end on a long one: round t lists, for every sequence that has that many, its
// t-th group from the end.
__global__ __launch_bounds__(1024) void sequence_worklist_kernel(const int32_t* __restrict__ cu_seq_new,
                                                                 const int32_t* __restrict__ seq_len, int B, int NQ,
                                                                 int qpg, int max_items, int32_t* __restrict__ plan) {
  __shared__ int ngr[ASPD_MAX_BATCH];
  __shared__ int first_item[ASPD_MAX_BATCH + 1];
  const int tid = threadIdx.x;
  // (a sequence that was refused holds no token: seq_len, which the kernel before this one wrote, says so,
  // while the packed rows the layout gave it stay where they are, unwritten)
  for (int s = tid; s < B; s += blockDim.x) ngr[s] = (max(seq_len[s], 0) + qpg - 1) / qpg;
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    for (int s = 0; s < B; ++s) {
      first_item[s] = acc;
      acc += ngr[s];
    }
    first_item[B] = min(acc, max_items);
    plan[0] = first_item[B];
    plan[1] = qpg;
    plan[2] = NQ;
    plan[3] = B;
    for (int i = 4; i < SEQ_PLAN_HDR; ++i) plan[i] = 0;
  }
  __syncthreads();
  const int n_items = first_item[B];
  int32_t* items = plan + SEQ_PLAN_HDR + ((NQ + 3) & ~3);
  // item (s, t): group ngr[s] - 1 - t of sequence s.  Its place in the list: the items of earlier rounds
  // (min(ngr, t) of every sequence) and, in its own round, the sequences before s that still have a group.
  for (int e = tid; e < n_items; e += blockDim.x) {
    int lo = 0, hi = B - 1;  // sequence of the e-th group in sequence-major order
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (first_item[mid] <= e) lo = mid; else hi = mid - 1;
    }
    const int s = lo;
    const int gidx = e - first_item[s];     // group index within the sequence, 0 = first tokens
    const int t = ngr[s] - 1 - gidx;
    int place = 0;
    for (int k = 0; k < B; ++k) place += min(ngr[k], t) + ((k < s && ngr[k] > t) ? 1 : 0);
    const int T = seq_len[s];
    const int tok0 = gidx * qpg;
    const int nq = min(qpg, T - tok0);
    if (place < n_items) {
      items[4 * place + 0] = s;
      items[4 * place + 1] = cu_seq_new[s] + tok0;
      items[4 * place + 2] = nq;
      items[4 * place + 3] = (tok0 + nq + ASPD_BLOCK - 1) / ASPD_BLOCK;  // pages up to the group's last slot
    }
  }
}

}  // namespace

size_t aspd_sequence_plan_words(const aspd_kv* kv, int32_t B, int32_t NQ) {
  const int G = kv->num_q_heads / kv->num_kv_heads;
  const int qpg = aspd_sequence_qpg(G);
  const size_t items = (size_t)B + (size_t)NQ / qpg;
  return (size_t)SEQ_PLAN_HDR + (((size_t)NQ + 3) & ~(size_t)3) + 4 * items;
}

extern "C" size_t aspd_sequence_plan_bytes(const aspd_kv* kv, int32_t B, int32_t NQ) {
  if (aspd_check_kv(kv) != ASPD_OK || B <= 0 || B > ASPD_MAX_BATCH || NQ < 0) return 0;
  const int G = kv->num_q_heads / kv->num_kv_heads;
  if (kv->dtype != ASPD_BF16 || aspd_sequence_qpg(G) < 1) return 0;
  return aspd_sequence_plan_words(kv, B, NQ) * sizeof(int32_t);
}

extern "C" int aspd_build_sequence_meta(const aspd_kv* kv, aspd_state* state, const aspd_layout* layout,
                                        int32_t pos_mode, aspd_step* out, void* stream) {
  int rc = aspd_check_kv(kv);
  if (rc != ASPD_OK) return rc;
  if (!state || !layout || !out || state->B <= 0 || !state->stage_base_d || !state->seq_len_d) return ASPD_ERR_INVALID_ARG;
  if (state->B > ASPD_MAX_BATCH) return ASPD_ERR_UNSUPPORTED;
  const int G = kv->num_q_heads / kv->num_kv_heads;
  if (kv->dtype != ASPD_BF16 || aspd_sequence_qpg(G) < 1) return ASPD_ERR_UNSUPPORTED;
  if (layout->num_runs < 0 || !layout->cu_runs_d || (layout->num_runs > 0 && (!layout->run_branch_d || !layout->run_len_d)))
    return ASPD_ERR_INVALID_ARG;
  const int mode = pos_mode & 0xff;
  const int fix_n = mode == 2 ? (pos_mode >> 8) : 0;
  if (mode < 0 || mode > 2 || (mode == 2 && fix_n <= 0)) return ASPD_ERR_INVALID_ARG;
  if (mode != ASPD_POS_SAME_SEQ && !state->main_pos_d) return ASPD_ERR_INVALID_ARG;
  if (state->slot_owner_d && state->owner_stride <= 0) return ASPD_ERR_INVALID_ARG;
  if (out->NQ < 0 || !out->cu_seq_new_d) return ASPD_ERR_INVALID_ARG;
  if (out->NQ > 0 && (!out->q_seq_d || !out->q_branch_d || !out->position_ids_d || !out->logical_slot_d ||
                      !out->slot_mapping_d || !out->kv_len_d))
    return ASPD_ERR_INVALID_ARG;
  if (!out->plan_d || ((uintptr_t)out->plan_d & 255) ||
      out->plan_bytes < aspd_sequence_plan_words(kv, state->B, out->NQ) * sizeof(int32_t))
    return ASPD_ERR_INVALID_ARG;
  hipStream_t hs = (hipStream_t)stream;
  const int qpg = aspd_sequence_qpg(G);
  LayoutView lay{layout->cu_runs_d, layout->run_branch_d, layout->run_len_d};
  hipLaunchKernelGGL(meta_sequence_kernel, dim3(state->B), dim3(SEQ_META_THREADS), 0, hs, make_view(kv), make_view(state),
                     make_view(out), lay, out->plan_d, mode == ASPD_POS_SAME_SEQ, mode == ASPD_POS_SAME_MAX, fix_n);
  ASPD_HIP_CHECK(hipGetLastError());
  const int max_items = state->B + out->NQ / qpg;
  hipLaunchKernelGGL(sequence_worklist_kernel, dim3(1), dim3(1024), 0, hs, out->cu_seq_new_d, state->seq_len_d, state->B,
                     out->NQ, qpg, max_items, out->plan_d);
  ASPD_HIP_CHECK(hipGetLastError());
  out->plan_key = aspd_sequence_plan_key(qpg, state->B);
  return ASPD_OK;
}
